"""End-to-end GPU parity of confspec_verify against the CPU oracle.

Small cases are compared on every trace; the full-size configurations run the GPU pass at full size
(the launch configuration the benchmark times) and compare a sample of traces the oracle can
compute in seconds - traces are independent, so a sampled trace checks the same code paths as any
other.  Bounds: see tests/gpu_cases.TOL.
"""
import numpy as np
import pytest
import torch

import confspec_workloads as W
from oracle import confspec_oracle as O
from paper_2602_18447_amd import binding as cb
from paper_2602_18447_amd.runner import Verifier
from tests import gpu_cases as G

pytestmark = pytest.mark.gpu


def test_config1_tiny_fp32_cache_from_prefix_pass():
    print("config 1", flush=True)
    wl = W.config(1)
    taus = [0.5, 0.52, 0.55, 0.6, 0.9]           # 0.9 alone is all-escalate at this width
    s, gpu, ora = G.parity_case(wl, taus=taus)
    assert s["traces"] == 4
    # cached suffix prefill on the GPU equals the oracle's full recompute over prefix + suffix
    weights, batch, kv = G.build_inputs(wl)
    model = W.OracleModelView(weights)
    pre = W.make_prefix_ids(wl)
    ids = batch.suffix_ids.cpu().numpy()
    e = np.zeros((0, wl.model.n_kv_heads, wl.model.head_dim))
    for b in range(wl.B):
        suf = ids[batch.h_cu_suffix[b]:batch.h_cu_suffix[b + 1]]
        xs, _ = O.forward(wl.model, model, [dict(ids=np.concatenate([pre[b], suf]), L=0,
                                                 k_prefix=lambda l: e, v_prefix=lambda l: e)])
        z = O.verdict_logits(xs[0][-1], model.final_norm, model.lm_head_rows(gpu["vids"]), wl.model.rms_eps)
        assert np.abs(gpu["logits"][b] - z).max() <= 1e-4


def _small_bf16(name, seed, prefix_lens, suffix_lens, **kw):
    base = dict(dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=768,
                vocab=1024, block_size=16, taus=(0.5, 0.55, 0.6, 0.9))
    base.update(kw)
    return W.tiny_workload(name, seed, prefix_lens=prefix_lens, suffix_lens=suffix_lens, **base)


def test_small_bf16_ragged_every_trace():
    print("small bf16 ragged", flush=True)
    wl = _small_bf16("small_ragged", 2001, (0, 5, 77, 300, 1, 1000, 130), (1, 7, 33, 64, 100, 96, 250))
    s, _, _ = G.parity_case(wl)
    assert s["traces"] == 7


def test_small_bf16_gqa6_cache_from_prefix_pass():
    """Draft-like head grouping (6 q heads per kv head); bf16 cache built by the oracle's prefix pass."""
    print("small bf16 gqa6 prefix-pass", flush=True)
    wl = _small_bf16("small_gqa6", 2002, (40, 129), (20, 70), n_q_heads=12, n_kv_heads=2, d_model=768,
                     d_ffn=1024, kv_source="prefix_pass", n_layers=2)
    G.parity_case(wl)


def test_edge_single_token_no_prefix_and_max_verdicts_and_taus():
    print("edge cases", flush=True)
    wl = _small_bf16("edge", 2003, (0,), (1,), n_verdict=8, taus=(0.0, 0.125, 0.13, 0.2, 0.5, 0.9, 0.99, 1.0))
    s, gpu, _ = G.parity_case(wl)
    assert gpu["accept"][0].all()
    wl = _small_bf16("edge_fp32", 2004, (0, 31), (1, 2), dtype="fp32", head_dim=64, n_kv_heads=4, d_model=256)
    G.parity_case(wl)


def test_results_are_run_to_run_identical_and_independent_of_batch_composition():
    print("determinism / batch independence", flush=True)
    wl = _small_bf16("det", 2005, (700, 64, 0, 3000), (40, 96, 20, 7))
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    a = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    b = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["accept"], b["accept"])
    # each trace alone: the attention planner cuts the key range into pieces that depend on the whole batch,
    # which moves the points where probabilities are rounded to bf16; the results agree to a fraction of the
    # bf16 tolerance, not bit for bit
    ids = batch.suffix_ids.cpu().numpy()
    for t in range(wl.B):
        one = W.tiny_workload("one", wl.seed, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2,
                              head_dim=128, d_ffn=768, vocab=1024, block_size=16, taus=wl.taus,
                              prefix_lens=(wl.prefix_lens[t],), suffix_lens=(wl.suffix_lens[t],))
        b1 = W.make_batch(one, G.DEV)
        lo, hi = batch.h_cu_suffix[t], batch.h_cu_suffix[t + 1]
        b1.suffix_ids = torch.as_tensor(ids[lo:hi]).to(G.DEV)
        nb = (wl.prefix_lens[t] + 15) // 16
        b1.block_table = batch.block_table[t:t + 1, :max(nb, 1)].contiguous()
        b1.n_blocks, b1.max_blocks_per_seq = batch.n_blocks, max(nb, 1)
        r = G.run_gpu(wl, weights, b1, kv, verifier=ver)
        assert np.abs(r["logits"][0] - a["logits"][t]).max() <= 6e-3
    ver.close()


def test_last_layer_pruning_changes_nothing_but_rounding():
    """The last layer computed for every row and for the last position of each trace only: same verdict
    logits up to the rounding differences of differently cut attention pieces."""
    print("last-layer pruning on / off", flush=True)
    wl = _small_bf16("prune", 2006, (700, 64, 0, 3000, 129), (40, 96, 20, 7, 1))
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    res = {}
    try:
        for flag in (0, 1):
            cb.confspec_tune(ver.ctx, "prune_last_layer", flag)
            res[flag] = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    finally:
        cb.confspec_tune(ver.ctx, "prune_last_layer", 1)
    assert np.abs(res[0]["logits"] - res[1]["logits"]).max() <= 6e-3
    ora = G.run_oracle(wl, weights, batch, kv, res[1]["taus"], res[1]["vids"])
    for flag in (0, 1):
        G.compare(wl, res[flag], ora, f"prune_last_layer={flag}")
    ver.close()


def test_first_layers_fp16_and_two_term_both_meet_the_bound():
    """The first layers' GEMMs on fp16 operands (default) or with two-term bf16 activations."""
    print("first layers: fp16 operands / two bf16 terms", flush=True)
    wl = _small_bf16("f16", 2007, (700, 64, 0, 3000, 129), (40, 96, 20, 7, 1), n_layers=8)
    weights, batch, kv = G.build_inputs(wl)
    res = {}
    try:
        for flag in (0, 1):
            cb.confspec_tune(None, "first_layers_f16", flag)     # default of new contexts: read when the weights are packed and by the pass
            ver = Verifier(wl.model, weights)
            assert ver.w.n_f16_layers == (4 if flag else 0)     # default: the first half of the 8 layers
            res[flag] = G.run_gpu(wl, weights, batch, kv, verifier=ver)
            ver.close()
    finally:
        cb.confspec_tune(None, "first_layers_f16", 1)
    ora = G.run_oracle(wl, weights, batch, kv, res[1]["taus"], res[1]["vids"])
    for flag in (0, 1):
        G.compare(wl, res[flag], ora, f"first_layers_f16={flag}")


def test_huge_activations_in_the_fp16_layers_give_finite_outputs():
    """Norm gains of about 1e5 in the layers that run on fp16 operands push normalised activations past the half
    range; they saturate there, and logits and confidences stay finite (no infinity, so no NaN downstream)."""
    print("fp16 layers with out-of-range activations", flush=True)
    wl = _small_bf16("huge", 2011, (300, 0, 64), (40, 7, 96), n_layers=4)
    weights, batch, kv = G.build_inputs(wl)
    for l in range(2):                                   # the first half of the layers: the fp16 ones
        weights.attn_norm[l].mul_(1.0e5)
        weights.mlp_norm[l].mul_(1.0e5)
    ver = Verifier(wl.model, weights)
    assert ver.w.n_f16_layers == 2
    r = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    ver.close()
    assert np.isfinite(r["logits"]).all() and np.isfinite(r["conf"]).all()
    assert np.all(r["conf"] >= 0.5 - 1e-6) and np.all(r["conf"] <= 1.0 + 1e-6)


def _shared_case(name, seed, groups, **kw):
    """groups: list of (prefix_len, [suffix lengths of the candidates]).  Returns workload, inputs with the candidates
    of a group reading their context through one set of pages, and the partition."""
    prefix, suffix, gstart = [], [], [0]
    for L, ss in groups:
        prefix += [L] * len(ss)
        suffix += list(ss)
        gstart.append(gstart[-1] + len(ss))
    wl = _small_bf16(name, seed, tuple(prefix), tuple(suffix), **kw)
    weights, batch, kv = G.build_inputs(wl)
    table = batch.block_table.clone()
    for lo, hi in zip(gstart[:-1], gstart[1:]):
        table[lo:hi] = table[lo]
    batch.block_table = table
    return wl, weights, batch, kv, gstart


@pytest.mark.parametrize("heads", [(12, 2), (4, 2)])
def test_candidates_on_a_shared_context_match_the_oracle(heads):
    """Section 4.3: the candidates of one step verified side by side on one context.  Groups of 2 and 4 candidates
    with short steps (a whole group inside one row tile), with 96-token steps (groups spanning several tiles, tiles
    spanning two candidates), ragged groups, and plain traces, in one batch; every trace against the oracle, and
    against the plain pass on the same batch."""
    hq, hkv = heads
    print(f"shared-context groups, heads {hq}/{hkv}", flush=True)
    groups = [(700, [5, 21, 1, 13]), (64, [96, 96]), (300, [50]), (1000, [40, 7, 130]), (0, [9, 3]), (129, [96, 96, 96, 96]),
              (33, [20, 21])]
    wl, weights, batch, kv, gstart = _shared_case("shared", 2012, groups, n_q_heads=hq, n_kv_heads=hkv,
                                                 d_model=128 * max(hq // 2, 2))
    ver = Verifier(wl.model, weights)
    vids = W.draw_verdict_ids(wl)
    taus = list(wl.taus)
    plain = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    outs = ver.verify_shared(kv, batch, gstart, vids, taus)
    torch.cuda.synchronize()
    shared = dict(logits=outs[0].cpu().numpy().astype(np.float64), conf=outs[1].cpu().numpy().astype(np.float64),
                  verdict=outs[2].cpu().numpy(), accept=outs[3].cpu().numpy(), taus=taus, vids=vids)
    ora = G.run_oracle(wl, weights, batch, kv, taus, vids)
    G.compare(wl, shared, ora, "shared-context groups")
    assert np.abs(shared["logits"] - plain["logits"]).max() <= 6e-3
    # the register-staged main loop on the same groups
    cb.confspec_tune(ver.ctx, "attn_kernel", 1)
    outs = ver.verify_shared(kv, batch, gstart, vids, taus)
    torch.cuda.synchronize()
    staged = dict(shared, logits=outs[0].cpu().numpy().astype(np.float64), conf=outs[1].cpu().numpy().astype(np.float64),
                  verdict=outs[2].cpu().numpy(), accept=outs[3].cpu().numpy())
    G.compare(wl, staged, ora, "shared-context groups, register-staged kernel")
    ver.close()


def test_both_attention_main_loops_meet_the_bound():
    print("attention main loops: software-pipelined / register-staged", flush=True)
    wl = _small_bf16("loops", 2013, (700, 64, 0, 3000, 129, 1, 1023), (40, 96, 20, 7, 1, 200, 64), n_layers=4)
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    res = {}
    for flag in (0, 1):
        cb.confspec_tune(ver.ctx, "attn_kernel", flag)
        res[flag] = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    ver.close()
    ora = G.run_oracle(wl, weights, batch, kv, res[0]["taus"], res[0]["vids"])
    for flag in (0, 1):
        G.compare(wl, res[flag], ora, f"attn_kernel={flag}")
    assert np.abs(res[0]["logits"] - res[1]["logits"]).max() <= 6e-3


def test_fused_and_separate_rotary_embedding_agree():
    print("rope in the projection epilogue / as a kernel of its own", flush=True)
    wl = _small_bf16("rope", 2008, (700, 64, 0, 3000, 129), (40, 96, 20, 7, 1), n_layers=8)
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    res = {}
    try:
        for flag in (0, 1):
            cb.confspec_tune(ver.ctx, "fuse_rope", flag)
            res[flag] = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    finally:
        cb.confspec_tune(ver.ctx, "fuse_rope", 1)
    ver.close()
    ora = G.run_oracle(wl, weights, batch, kv, res[1]["taus"], res[1]["vids"])
    for flag in (0, 1):
        G.compare(wl, res[flag], ora, f"fuse_rope={flag}")


def test_weight_prefetch_hint_changes_no_bit():
    print("down-projection weight prefetch on / off", flush=True)
    wl = _small_bf16("prefetch", 2009, (700, 64, 0, 3000, 129), (40, 96, 20, 7, 1), n_layers=6, d_ffn=2048)
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    res = {}
    try:
        for flag in (0, 1):
            cb.confspec_tune(ver.ctx, "prefetch_down", flag)
            res[flag] = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    finally:
        cb.confspec_tune(ver.ctx, "prefetch_down", 1)
    ver.close()
    for k in ("logits", "conf", "verdict", "accept"):
        assert np.array_equal(res[0][k], res[1][k])


def _full_size(cfg, traces):
    """Full-size GPU pass (the launch configuration the benchmark times) against the oracle on sampled traces, with
    the threshold sweep; both gate outcomes must occur among the compared decisions."""
    wl = W.config(cfg)
    s, gpu, _ = G.parity_case(wl, traces=traces, taus=G.sweep_taus(wl))
    assert s["traces"] == len(traces)
    assert s["gate_kept"] > 0 and s["gate_escalated"] > 0, s
    return s, gpu


def test_config2_draft_shape_full_size_sampled_traces():
    print("config 2", flush=True)
    _full_size(2, [0, 7, 13, 22, 31])


def test_config3_long_cot_tau_sweep_sampled_traces():
    print("config 3", flush=True)
    s, gpu = _full_size(3, [0, 5, 7, 21, 33, 40, 63])
    assert {0.8, 0.9, 0.95} <= set(gpu["taus"])


def test_config4_ragged_sampled_traces():
    print("config 4", flush=True)
    wl = W.config(4)
    L = np.asarray(wl.prefix_lens)
    S = np.asarray(wl.suffix_lens)
    pick = sorted({int(np.argmin(L)), int(np.argmax(L)), int(np.argmin(S)), int(np.argmax(S)), 3, 40, 77, 101, 127})
    assert len(pick) >= 8
    _full_size(4, pick)


def test_config5_target_shape_sampled_traces():
    print("config 5", flush=True)
    _full_size(5, [0, 4, 9, 15])


@pytest.mark.parametrize("seed", [3101, 3102, 3103, 3104, 3105, 3106])
def test_seeded_random_small_batches(seed):
    """Random head groupings, batch sizes and lengths (context lengths on and around page and chunk borders,
    single-token suffixes, empty contexts), every trace against the oracle."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    hq, hkv = [(4, 2), (12, 2), (8, 8), (6, 1), (8, 4), (10, 2)][seed % 6]
    B = int(rng.integers(1, 9))
    special = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024]
    L = [int(rng.choice(special)) if rng.random() < 0.5 else int(rng.integers(0, 1500)) for _ in range(B)]
    S = [1 if rng.random() < 0.2 else int(rng.integers(1, 200)) for _ in range(B)]
    n_layers = int(rng.integers(1, 5))
    print(f"random small batch seed={seed}: heads {hq}/{hkv}, layers {n_layers}, L={L}, S={S}", flush=True)
    wl = _small_bf16(f"rand{seed}", seed, tuple(L), tuple(S), n_q_heads=hq, n_kv_heads=hkv, d_model=128 * max(hq // 2, 2),
                     d_ffn=int(rng.choice([512, 768, 1280])), n_layers=n_layers)
    s, _, _ = G.parity_case(wl)
    assert s["traces"] == B


def test_hip_graph_replays_match_eager_results():
    """The pass captured once into a HIP graph: several replays, with eager passes on other inputs and
    synchronisations in between, each give the eager result of their inputs bit for bit."""
    print("graph capture / replay", flush=True)
    wl = _small_bf16("graph", 2010, (700, 64, 0, 3000, 129), (40, 96, 20, 7, 1), n_layers=4)
    weights, batch, kv = G.build_inputs(wl)
    vids = W.draw_verdict_ids(wl)
    taus = list(wl.taus)
    ver = Verifier(wl.model, weights)
    outs = ver.alloc_outputs(wl.B, len(vids), len(taus))
    ver.verify(kv, batch, vids, taus, outputs=outs)
    torch.cuda.synchronize()
    eager = [t.clone() for t in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ver.verify(kv, batch, vids, taus, outputs=outs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ver.verify(kv, batch, vids, taus, outputs=outs)
    # a second set of suffix ids, written into the captured input buffer between replays
    ids_a = batch.suffix_ids.clone()
    ids_b = torch.roll(ids_a, 5)
    batch.suffix_ids.copy_(ids_b)
    ver2 = Verifier(wl.model, weights)
    eager_b = [t.clone() for t in ver2.verify(kv, batch, vids, taus)]
    torch.cuda.synchronize()
    for i in range(6):
        use_b = i % 2 == 1
        batch.suffix_ids.copy_(ids_b if use_b else ids_a)
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        want = eager_b if use_b else eager
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), (i, use_b)
        ver2.verify(kv, batch, vids, taus)                 # eager work of the same library between replays
        torch.cuda.synchronize()
    ver.close()
    ver2.close()
