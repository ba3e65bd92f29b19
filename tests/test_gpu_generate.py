"""GPU parity of the generation step (the pass + the full-vocabulary head) and of greedy generation on a growing
cache against the CPU oracle.  Bounds: max logit and log-sum-exp within the logit bound of tests/gpu_cases.TOL, the
full-vocabulary confidence within the confidence bound, the token equal wherever the oracle's arg max leads the
runner-up by more than twice the logit bound (below that both precisions may legitimately pick either)."""
import numpy as np
import pytest
import torch

import confspec_workloads as W
from oracle import confspec_oracle as O
from paper_2602_18447_amd import binding as cb
from paper_2602_18447_amd.runner import Verifier
from tests import gpu_cases as G

pytestmark = pytest.mark.gpu
DEV = G.DEV


def _compare_step(dtype, gpu, ora, label):
    tol = G.TOL[dtype]
    tr = ora["traces"]
    g = {k: v.cpu().numpy() for k, v in gpu.items()}
    d_max = np.abs(g["max_logit"][tr] - ora["max_logit"]).max()
    d_lse = np.abs(g["lse"][tr] - ora["lse"]).max()
    decided = ora["margin"] > 2 * tol["logit"]
    mism = int((g["token"][tr][decided] != ora["token"][decided]).sum())
    print(f"{label}: traces {len(tr)}, decided {int(decided.sum())}, |d max_logit| {d_max:.2e}, |d lse| {d_lse:.2e}, "
          f"token mismatches {mism}", flush=True)
    assert d_max <= tol["logit"] and d_lse <= tol["logit"] and mism == 0
    assert np.all(g["max_logit"] <= g["lse"] + 1e-6)
    if "conf_full" in ora:
        assert np.abs(g["conf_full"][tr] - ora["conf_full"]).max() <= tol["conf"]
    return decided


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_generation_step_matches_oracle_on_a_ragged_batch(dtype):
    print(f"generation step {dtype}", flush=True)
    kw = dict(vocab=1024, block_size=16, prefix_lens=(0, 5, 77, 300, 16, 1000, 130), suffix_lens=(1, 7, 1, 64, 100, 1, 33))
    if dtype == "bf16":
        wl = W.tiny_workload("gen", 6100, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128,
                             d_ffn=768, **kw)
    else:
        wl = W.tiny_workload("gen32", 6101, dtype="fp32", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                             d_ffn=512, **kw)
    weights, batch, kv = G.build_inputs(wl)
    vids = W.draw_verdict_ids(wl)
    ver = Verifier(wl.model, weights)
    ora = O.next_token(wl.model, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                       batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, verdict_ids=vids)
    gpu = ver.generate_step(kv, batch, verdict_ids=vids)
    torch.cuda.synchronize()
    _compare_step(dtype, gpu, ora, f"step {dtype}")
    # without verdict tokens: same token statistics, bit for bit
    plain = ver.generate_step(kv, batch)
    torch.cuda.synchronize()
    for k in ("token", "max_logit", "lse"):
        assert torch.equal(plain[k], gpu[k])
    # the restricted confidence of the plain pass is the full-vocabulary one renormalised over the verdict tokens
    logits, conf, _, _ = ver.verify(kv, batch, vids, [0.5])
    torch.cuda.synchronize()
    p_full = torch.exp(logits - gpu["lse"][:, None])
    assert torch.allclose(p_full.max(dim=1).values, gpu["conf_full"], rtol=1e-5, atol=1e-7)
    assert torch.allclose(p_full.max(dim=1).values / p_full.sum(dim=1), conf, rtol=1e-4, atol=1e-6)
    # argument errors
    with pytest.raises(cb.ConfSpecError):
        ho = cb.HeadOut(gpu["token"].data_ptr(), gpu["max_logit"].data_ptr(), gpu["lse"].data_ptr(), None)
        kvs, bs, keep = ver.bind(kv, batch)
        cb.confspec_generate_step(ver.ctx, ver.w, kvs, bs, None, None, None, ver.workspace(bs.T, bs.B),
                                  torch.empty(256, dtype=torch.uint8, device=DEV), ho)
    ver.close()


def test_greedy_generation_on_a_growing_cache_matches_oracle():
    print("greedy generation", flush=True)
    n_steps = 6
    ctx_len = (40, 1, 129, 16, 3, 64, 255, 17, 90, 33)
    wl = W.tiny_workload("greedy", 6200, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128,
                         d_ffn=768, vocab=1024, block_size=16, prefix_lens=ctx_len, suffix_lens=(1,) * len(ctx_len),
                         kv_source="prefix_pass")
    weights = W.make_weights(wl.model, wl.seed, DEV)
    batch = W.make_batch(wl, DEV, extra_rows=n_steps)
    model = W.OracleModelView(weights)
    kd, vd = O.prefix_pass(wl.model, model, W.make_prefix_ids(wl))
    kv = W.pages_from_dense(wl, batch, kd, vd, DEV)
    view = W.OracleKVView(kv, batch)
    table = batch.block_table.cpu().numpy()
    k_ctx = [[O.gather_prefix(view.k_blocks(l, table[b, :(L + 15) // 16]), L) for b, L in enumerate(ctx_len)]
             for l in range(wl.model.n_layers)]                 # the rounded values the GPU reads
    v_ctx = [[O.gather_prefix(view.v_blocks(l, table[b, :(L + 15) // 16]), L) for b, L in enumerate(ctx_len)]
             for l in range(wl.model.n_layers)]
    first = batch.suffix_ids.cpu().numpy()
    toks_o, zmax_o, lse_o, k_o, v_o, margin = O.generate_greedy(wl.model, model, k_ctx, v_ctx, first, n_steps, want_margin=True)
    ver = Verifier(wl.model, weights)
    toks, zmax, lse = ver.generate_greedy(kv, batch.block_table, batch.n_blocks, batch.max_blocks_per_seq,
                                          batch.suffix_ids, batch.h_prefix_lens, n_steps)
    torch.cuda.synchronize()
    toks, zmax, lse = toks.cpu().numpy().T, zmax.cpu().numpy().T, lse.cpu().numpy().T       # [B, n_steps]
    tol = G.TOL["bf16"]
    followed = 0
    for b in range(wl.B):
        for i in range(n_steps):
            assert abs(zmax[b, i] - zmax_o[b, i]) <= tol["logit"] and abs(lse[b, i] - lse_o[b, i]) <= tol["logit"], (b, i)
            if toks[b, i] != toks_o[b, i]:
                assert margin[b, i] <= 2 * tol["logit"], (b, i)   # only an undecided arg max may differ;
                break                                             # from here on the two sides follow different tokens
            followed += 1
        else:
            # the whole continuation agreed: the rows the GPU appended are the oracle's
            L = ctx_len[b]
            for l in range(wl.model.n_layers):
                for pages, ref in ((kv.k_pages, k_o[l][b]), (kv.v_pages, v_o[l][b])):
                    got = np.stack([pages[l][int(table[b, j // 16]), :, j % 16, :].to(torch.float64).cpu().numpy()
                                    for j in range(L, L + n_steps)])
                    assert np.abs(got - ref[L:]).max() <= 2e-2 * np.abs(ref[L:]).max()
    print(f"greedy generation: both sides on the same continuation for {followed} of {wl.B * n_steps} steps", flush=True)
    assert followed >= 0.7 * wl.B * n_steps
    ver.close()


def test_decode_step_full_size_draft_shape_sampled_traces():
    print("decode step, draft shape B=32 L=2048", flush=True)
    m = W.DRAFT_SHAPE
    wl = W.Workload("decode_b32_L2048", m, 1022, (2048,) * 32, (1,) * 32)
    weights = W.make_weights(m, wl.seed, DEV)
    batch = W.make_batch(wl, DEV, extra_rows=1)
    kv = W.make_seeded_kv(wl, batch, DEV)
    vids = W.draw_verdict_ids(wl)
    ver = Verifier(m, weights)
    sample = [0, 17, 31]
    ora = O.next_token(m, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                       batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, verdict_ids=vids,
                       trace_subset=sample)
    gpu = ver.generate_step(kv, batch, n_append=np.ones(32, dtype=np.int32), verdict_ids=vids)
    torch.cuda.synchronize()
    _compare_step("bf16", gpu, ora, "decode step config-2 shape")
    ver.close()
