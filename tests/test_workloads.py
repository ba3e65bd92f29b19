"""The synthetic-input recipe: shapes, determinism, paging, and the oracle driven through it."""
import numpy as np
import torch

import confspec_workloads as W
from oracle import confspec_oracle as O


def test_five_configs_have_the_stated_shapes():
    c1, c2, c3, c4, c5 = (W.config(i) for i in range(1, 6))
    assert (c1.model.dtype, c1.B, c1.T, c1.model.n_layers, c1.model.group) == ("fp32", 4, 128, 2, 1)
    assert (c2.B, c2.T, c2.model.qkv_rows, c2.model.d_ffn) == (32, 3072, 2048, 8960)
    assert (c3.B, c3.T, c3.taus) == (64, 8192, (0.8, 0.9, 0.95))
    assert c4.B == 128 and min(c4.prefix_lens) >= 512 and max(c4.prefix_lens) <= 16384
    assert min(c4.suffix_lens) >= 32 and max(c4.suffix_lens) <= 256
    assert c4 == W.config(4)                       # ragged lengths are a pure function of the seed
    assert (c5.model.n_layers, c5.model.d_model, c5.model.group, c5.T) == (64, 5120, 5, 1536)
    for c in (c2, c3, c4, c5):
        assert c.block_size == 16 and c.model.dtype == "bf16" and c.model.rope_theta == 1e6


def test_generation_is_seeded_and_rounded_to_storage_dtype():
    wl = W.tiny_workload("t", 5, dtype="bf16")
    a, b = W.make_weights(wl.model, wl.seed), W.make_weights(wl.model, wl.seed)
    assert torch.equal(a.wqkv[1], b.wqkv[1]) and a.wqkv[0].dtype == torch.bfloat16
    assert not torch.equal(a.wqkv[0], a.wqkv[1])
    assert not torch.equal(a.embed, W.make_weights(wl.model, wl.seed + 1).embed)
    assert abs(float(a.attn_norm[0].float().mean()) - 1.0) < 0.02
    assert 0.015 < float(a.w_down[0].float().std()) < 0.025


def test_block_table_is_a_partial_permutation_and_pages_round_trip():
    wl = W.tiny_workload("t", 6, prefix_lens=(5, 0, 19, 8), suffix_lens=(3, 1, 7, 2))
    batch = W.make_batch(wl)
    need = [(L + 3) // 4 for L in wl.prefix_lens]
    used = np.concatenate([batch.block_table[b, :n].numpy() for b, n in enumerate(need)])
    assert len(set(used.tolist())) == len(used) and used.max() < batch.n_blocks
    assert list(batch.h_cu_suffix) == [0, 3, 4, 11, 13]
    rng = np.random.default_rng(0)
    m = wl.model
    kd = [[rng.normal(0, 1, (L, m.n_kv_heads, m.head_dim)) for L in wl.prefix_lens] for _ in range(m.n_layers)]
    kv = W.pages_from_dense(wl, batch, kd, kd)
    view = W.OracleKVView(kv, batch)
    for b, L in enumerate(wl.prefix_lens):
        if L == 0:
            continue
        rows = O.gather_prefix(view.k_blocks(1, batch.block_table[b, :need[b]].numpy()), L)
        np.testing.assert_allclose(rows, kd[1][b].astype(np.float32), rtol=0, atol=0)


def test_config1_cache_from_prefix_pass_matches_full_recompute():
    """fp32 pages built from the oracle's own prefix pass: cached prefill == recompute
    up to the fp32 rounding of the stored K/V."""
    wl = W.tiny_workload("c1_small", 1001, dtype="fp32", n_layers=2, d_model=64, n_q_heads=4,
                         n_kv_heads=4, head_dim=16, d_ffn=128, vocab=211, prefix_lens=(17, 9),
                         suffix_lens=(5, 3), block_size=16, kv_source="prefix_pass")
    w = W.make_weights(wl.model, wl.seed, std=0.2)
    model = W.OracleModelView(w)
    batch = W.make_batch(wl)
    pre = W.make_prefix_ids(wl)
    kd, vd = O.prefix_pass(wl.model, model, pre)
    kv = W.pages_from_dense(wl, batch, kd, vd)
    vids = W.draw_verdict_ids(wl)
    res = O.verify(wl.model, model, W.OracleKVView(kv, batch), 16, batch.suffix_ids.numpy(),
                   batch.h_cu_suffix, batch.h_prefix_lens, vids, wl.taus)
    e = np.zeros((0, 4, 16))
    for b in range(wl.B):
        suf = batch.suffix_ids.numpy()[batch.h_cu_suffix[b]:batch.h_cu_suffix[b + 1]]
        xs, _ = O.forward(wl.model, model, [dict(ids=np.concatenate([pre[b], suf]), L=0,
                                                 k_prefix=lambda l: e, v_prefix=lambda l: e)])
        z = O.verdict_logits(xs[0][-1], model.final_norm, model.lm_head_rows(vids), wl.model.rms_eps)
        np.testing.assert_allclose(res["logits"][b], z, rtol=0, atol=2e-5)


def test_random_init_gate_statistics_are_not_degenerate():
    """At N(0, 0.02) init the logit gap is roughly N(0, 2 * 0.02^2 * d): most confidences sit
    near 1/2, so gate tests need low thresholds as well as the paper's 0.9."""
    wl = W.tiny_workload("stat", 77, dtype="bf16", n_layers=1, d_model=256, n_q_heads=2, n_kv_heads=1,
                         head_dim=128, d_ffn=256, vocab=512, prefix_lens=(8,) * 24, suffix_lens=(4,) * 24,
                         block_size=16, taus=(0.5, 0.52, 0.55, 0.6, 0.9))
    w = W.make_weights(wl.model, wl.seed)
    batch = W.make_batch(wl)
    kv = W.make_seeded_kv(wl, batch)
    res = O.verify(wl.model, W.OracleModelView(w), W.OracleKVView(kv, batch), 16,
                   batch.suffix_ids.numpy(), batch.h_cu_suffix, batch.h_prefix_lens,
                   W.draw_verdict_ids(wl), wl.taus)
    acc = res["accept"].sum(axis=1)
    assert acc[0] == 24 and acc[-1] == 0 and list(acc) == sorted(acc, reverse=True)
    assert 0 < acc[2] < 24
