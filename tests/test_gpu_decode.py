"""GPU parity of passes with one new token per trace (generation steps; Algorithm 1's generate calls), which a bf16
context runs on kernels of their own: element-wise comparison of the verdict logits / confidences with the CPU oracle
on contexts around every border the kernels have (empty context, page, 256-key piece, one and 32 traces), on a model
whose k ranges are cut into slices, with the same batch on the general kernels beside it, and on the library's static
scratch."""
import numpy as np
import pytest
import torch

import confspec_workloads as W
from paper_2602_18447_amd import binding as cb
from paper_2602_18447_amd.runner import Verifier
from tests import gpu_cases as G

pytestmark = pytest.mark.gpu

TAUS = (0.5, 0.52, 0.55, 0.6, 0.9)


def _wl(name, seed, prefix_lens, **kw):
    args = dict(dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=768, vocab=1024,
                block_size=16, taus=TAUS, prefix_lens=prefix_lens, suffix_lens=(1,) * len(prefix_lens))
    args.update(kw)
    return W.tiny_workload(name, seed, **args)


def _run(wl, decode_kernels=1):
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    cb.confspec_tune(ver.ctx, "decode_kernels", decode_kernels)
    gpu = G.run_gpu(wl, weights, batch, kv, verifier=ver)
    ver.close()
    return weights, batch, kv, gpu


@pytest.mark.parametrize("case", ["borders", "one_trace", "32_traces", "from_prefix_pass", "long_contexts", "longer_contexts"])
def test_one_token_batches_match_oracle(case):
    print(f"one-token batch: {case}", flush=True)
    if case == "borders":
        wl = _wl("dec_borders", 7101, (0, 1, 15, 16, 17, 255, 256, 257, 511, 512, 513, 300, 1000))
    elif case == "one_trace":
        wl = _wl("dec_one", 7102, (777,))
    elif case == "32_traces":
        rng = np.random.default_rng(7103)
        wl = _wl("dec_32", 7103, tuple(int(v) for v in rng.integers(0, 700, 32)))
    elif case == "long_contexts":      # enough (trace, kv head, 256-key piece) triples that a workgroup makes 2 rounds of 256 keys
        rng = np.random.default_rng(7107)
        wl = _wl("dec_long", 7107, tuple(int(v) for v in rng.integers(2000, 4500, 24)) + (511, 512, 513, 1023, 1024, 0))
    elif case == "longer_contexts":    # ... 4 rounds
        rng = np.random.default_rng(7108)
        wl = _wl("dec_longer", 7108, tuple(int(v) for v in rng.integers(3000, 9000, 30)) + (1023, 1024), n_layers=2)
    else:
        wl = _wl("dec_ctx", 7104, (40, 1, 129, 16, 3, 64, 255, 17), kv_source="prefix_pass")
    weights, batch, kv, gpu = _run(wl)
    ora = G.run_oracle(wl, weights, batch, kv, gpu["taus"], gpu["vids"])
    s = G.compare(wl, gpu, ora, wl.name)
    assert s["traces"] == wl.B
    # the same batch on the general kernels: also the oracle's result, by a different arithmetic
    _, _, _, ref = _run(wl, decode_kernels=0)
    G.compare(wl, ref, ora, wl.name + " (general kernels)")
    assert not np.array_equal(ref["logits"], gpu["logits"]), "both settings produced the same bits: the step kernels did not run"
    assert np.abs(ref["logits"] - gpu["logits"]).max() <= 2 * G.TOL["bf16"]["logit"]


def test_one_token_batch_on_a_model_with_sliced_k_ranges():
    # d_model 2048 = 32 k-tiles: every projection's k range is cut into slices whose partial planes the last workgroup
    # to arrive adds up; 8 q heads per kv head (the most the step's attention takes).  Models this wide take the step
    # kernels only when asked to (setting 2).
    print("one-token batch, d_model 2048, 16 / 2 heads", flush=True)
    wl = _wl("dec_wide", 7105, (0, 33, 256, 700, 90), n_layers=2, d_model=2048, n_q_heads=16, n_kv_heads=2, d_ffn=2560)
    _, _, _, auto = _run(wl, decode_kernels=1)
    weights, batch, kv, gpu = _run(wl, decode_kernels=2)
    ora = G.run_oracle(wl, weights, batch, kv, gpu["taus"], gpu["vids"])
    G.compare(wl, gpu, ora, wl.name)
    _, _, _, ref = _run(wl, decode_kernels=0)
    assert not np.array_equal(ref["logits"], gpu["logits"])
    assert np.array_equal(ref["logits"], auto["logits"])      # the default leaves this model on the general kernels


def test_one_token_batch_is_repeatable_and_runs_on_the_static_scratch():
    print("one-token batch: two runs bit-identical; static scratch", flush=True)
    wl = _wl("dec_static", 7106, (700, 64, 0, 300, 129, 1000, 256, 31))
    weights, batch, kv = G.build_inputs(wl)
    ver = Verifier(wl.model, weights)
    vids = W.draw_verdict_ids(wl)
    a = [t.clone() for t in ver.verify(kv, batch, vids, list(TAUS))]
    b = [t.clone() for t in ver.verify(kv, batch, vids, list(TAUS))]
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)          # partial results are added in a fixed order, whoever adds them
    need = cb.confspec_static_scratch_need(ver.ctx, ver.bind(kv, batch)[1])
    assert need <= cb.STATIC_SCRATCH_BYTES
    outs = ver.alloc_outputs(wl.B, len(vids), len(TAUS))
    ver.verify_static(kv, batch, vids, list(TAUS), outs)
    torch.cuda.synchronize()
    for x, y in zip(a, outs):
        assert torch.equal(x, y)
    ver.close()
