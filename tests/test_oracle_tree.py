"""Pins of the oracle's tree walk (Section 4.3, Eq. 5): a chain is the linear cascade; one layer is an argmax over
the accepted candidates; random small trees against an independently written recursive form."""
import itertools

import numpy as np

from oracle import confspec_oracle as O


def _recursive(parent, v, p, cur=-1):
    """Chosen path below node cur, by recursion on a children table: best accepted child by (confidence, -index)."""
    kids = [j for j, q in enumerate(parent) if q == cur and v[j] == 0]
    if not kids:
        return []
    best = max(kids, key=lambda j: (p[j], -j))
    return [best] + _recursive(parent, v, p, best)


def test_chain_is_the_linear_cascade():
    gamma = 0.9
    for k in range(1, 5):
        parent = [-1] + list(range(k - 1))
        for rd in itertools.product((0, 1), repeat=k):
            for hi in itertools.product((0, 1), repeat=k):
                for rt in itertools.product((0, 1), repeat=k):
                    conf = [0.97 if h else 0.61 for h in hi]
                    m, dec, esc = O.cascade_request(rd, conf, lambda j: rt[j], gamma)
                    path, dec2, esc2, used = O.tree_request(parent, rd, conf, lambda j: (rt[j], 0.8), gamma)
                    assert path == list(range(m)) and list(dec) == list(dec2) and list(esc) == list(esc2)


def test_one_layer_selects_the_most_confident_accepted_candidate():
    parent = [-1, -1, -1, -1]
    # kept decisions: candidate 1 accepted at 0.93, candidate 3 accepted at 0.97; candidate 0 rejected with 0.99
    path, dec, esc, used = O.tree_request(parent, [1, 0, 0, 0], [0.99, 0.93, 0.5, 0.97], lambda j: (0, 0.95), 0.9)
    assert path == [3] and dec == [1, 0, 0, 0] and esc == [0, 0, 1, 0]
    assert used[2] == 0.95                                  # the large model's confidence enters the selection
    # ... and wins when it is the highest
    path, _, _, _ = O.tree_request(parent, [1, 0, 0, 0], [0.99, 0.93, 0.5, 0.94], lambda j: (0, 0.95), 0.9)
    assert path == [2]
    # ties go to the lowest index; nothing accepted: empty path, every candidate of the layer still decided
    assert O.tree_request(parent, [0, 0, 0, 0], [0.95] * 4, lambda j: (1, 1.0), 0.9)[0] == [0]
    path, dec, esc, used = O.tree_request(parent, [1, 1, 0, 1], [0.95, 0.95, 0.2, 0.95], lambda j: (1, 0.7), 0.9)
    assert path == [] and dec == [1, 1, 1, 1] and esc == [0, 0, 1, 0]


def test_random_trees_match_the_recursive_form_and_consult_lazily():
    rng = np.random.default_rng(11)
    for trial in range(400):
        n = int(rng.integers(1, 9))
        parent = [-1] + [int(rng.integers(-1, j)) for j in range(1, n)]
        rd = rng.integers(0, 2, size=n)
        rt = rng.integers(0, 2, size=n)
        pd = np.round(rng.uniform(0.5, 1.0, size=n), 2)
        pt = np.round(rng.uniform(0.5, 1.0, size=n), 2)
        gamma = float(rng.choice([0.0, 0.7, 0.9, 1.01]))
        asked = []
        path, dec, esc, used = O.tree_request(parent, rd, pd, lambda j: (asked.append(j), (rt[j], pt[j]))[1], gamma)
        keep = pd >= gamma
        v = np.where(keep, rd, rt)
        p = np.where(keep, pd, pt)
        want = _recursive(parent, v, p)
        assert path == want, (parent, list(v), list(p))
        on_path = [-1] + want
        reached = np.array([parent[j] in on_path[:len(want) + 1] and _is_live(parent, j, want) for j in range(n)])
        assert [d != O.NOT_REACHED for d in dec] == list(reached)
        assert list(np.asarray(dec)[reached]) == list(v[reached])
        assert sorted(asked) == [j for j in range(n) if reached[j] and not keep[j]] and list(esc) == [int(reached[j] and not keep[j]) for j in range(n)]
        assert np.array_equal(np.asarray(used)[reached], p[reached]) and np.isnan(np.asarray(used)[~reached]).all()


def _is_live(parent, j, path):
    """A node is looked at iff its parent is the root or a chosen node."""
    return parent[j] == -1 or parent[j] in path


def test_cascade_verify_on_a_forest_matches_the_recursive_form_on_full_batch_results():
    import confspec_workloads as W
    L, S = (5, 5, 5, 9, 9, 12, 3, 3), (4, 3, 6, 2, 5, 1, 3, 2)
    wl_d = W.tiny_workload("tree_d", 81, dtype="fp32", n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=32,
                           d_ffn=128, vocab=97, prefix_lens=L, suffix_lens=S)
    wl_t = W.tiny_workload("tree_t", 82, dtype="fp32", n_layers=2, d_model=96, n_q_heads=2, n_kv_heads=2, head_dim=48,
                           d_ffn=160, vocab=97, prefix_lens=L, suffix_lens=S)
    batch = W.make_batch(wl_d, "cpu")
    sides = []
    for wl in (wl_d, wl_t):
        weights = W.make_weights(wl.model, wl.seed, "cpu")
        kv = W.make_seeded_kv(wl, batch, "cpu")
        sides.append(dict(cfg=wl.model, model=W.OracleModelView(weights), kv=W.OracleKVView(kv, batch)))
    vids = W.draw_verdict_ids(wl_d)
    ids, cu, pl = batch.suffix_ids.numpy(), batch.h_cu_suffix, batch.h_prefix_lens
    req_start = [0, 6, 8]
    parent = [-1, -1, -1, 0, 0, 3, -1, -1]                  # request 0: three candidates, two below the first, one below that
    full = [O.verify(s["cfg"], s["model"], s["kv"], wl_d.block_size, ids, cu, pl, vids, [0.5]) for s in sides]
    for gamma in (0.0, 0.53, 0.6, 2.0):
        r = O.cascade_verify(sides[0], sides[1], wl_d.block_size, ids, cu, pl, vids, gamma, req_start, parent=parent)
        keep = full[0]["conf"] >= gamma
        v = np.where(keep, full[0]["verdict"], full[1]["verdict"])
        p = np.where(keep, full[0]["conf"], full[1]["conf"])
        for q, (lo, hi) in enumerate(zip(req_start[:-1], req_start[1:])):
            local = [parent[b] - lo if parent[b] >= 0 else -1 for b in range(lo, hi)]
            want = _recursive(local, v[lo:hi], p[lo:hi])
            assert r["accepted_steps"][q] == len(want)
            assert list(np.flatnonzero(r["selected"][lo:hi])) == sorted(want)
        asked = ~np.isnan(r["conf_target"])
        assert np.array_equal(asked, r["escalated"].astype(bool))
        reached = r["decision"] != O.NOT_REACHED
        assert np.allclose(r["conf_used"][reached], p[reached], atol=1e-12) and np.array_equal(r["decision"][reached], v[reached])
