"""The pass on the library's own scratch array (confspec_verify_static) against confspec_verify with a caller
workspace: same kernels, so the outputs must be bit-identical; two calls in a row on the shared array, the second
on a smaller batch; sizes beyond the array are refused before anything is launched."""
import numpy as np
import pytest
import torch

import confspec_workloads as W
from paper_2602_18447_amd import binding as cb
from paper_2602_18447_amd.runner import Verifier
from tests import gpu_cases as G

pytestmark = pytest.mark.gpu


def _wl(name, seed, prefix_lens, suffix_lens):
    return W.tiny_workload(name, seed, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128,
                           d_ffn=768, vocab=1024, block_size=16, taus=(0.5, 0.55, 0.6, 0.9),
                           prefix_lens=prefix_lens, suffix_lens=suffix_lens)


def test_static_scratch_pass_equals_workspace_pass_on_two_calls_in_a_row():
    print("no-allocation entry point: large batch, then a smaller one", flush=True)
    big = _wl("static_big", 5001, (700, 64, 0, 3000, 129, 1000), (40, 96, 20, 7, 1, 250))
    small = _wl("static_small", 5001, (64, 3000), (96, 7))
    weights = W.make_weights(big.model, big.seed, G.DEV)
    ver = Verifier(big.model, weights)
    vids = W.draw_verdict_ids(big)
    taus = list(big.taus)
    cases = []
    for wl in (big, small):
        batch = W.make_batch(wl, G.DEV)
        kv = W.make_seeded_kv(wl, batch, G.DEV)
        ref = [t.clone() for t in ver.verify(kv, batch, vids, taus)]
        torch.cuda.synchronize()
        need = cb.confspec_static_scratch_need(ver.ctx, ver.bind(kv, batch)[1])
        print(f"  {wl.name}: {need} bytes of scratch needed", flush=True)
        assert need <= cb.STATIC_SCRATCH_BYTES
        cases.append((wl, batch, kv, ref))
    # the two calls on the shared array, back to back on one stream, outputs preallocated
    outs = [ver.alloc_outputs(wl.B, len(vids), len(taus)) for wl, _, _, _ in cases]
    for o in outs:
        for t in o:
            t.fill_(7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (wl, batch, kv, _), o in zip(cases, outs):
        ver.verify_static(kv, batch, vids, taus, o)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for (wl, _, _, ref), o in zip(cases, outs):
        for got, want in zip(o, ref):
            assert torch.equal(got, want), wl.name
    # and the result is the oracle's, to the usual bound (first batch)
    wl, batch, kv, _ = cases[0]
    gpu = dict(logits=outs[0][0].cpu().numpy().astype(np.float64), conf=outs[0][1].cpu().numpy().astype(np.float64),
               verdict=outs[0][2].cpu().numpy(), accept=outs[0][3].cpu().numpy(), taus=taus, vids=vids)
    G.compare(wl, gpu, G.run_oracle(wl, weights, batch, kv, taus, vids), "static scratch")
    ver.close()


def test_static_scratch_refuses_batches_beyond_its_size():
    print("no-allocation entry point: size limit", flush=True)
    wl = _wl("static_limit", 5002, (16,), (8,))
    weights = W.make_weights(wl.model, wl.seed, G.DEV)
    ver = Verifier(wl.model, weights)
    T = 1 << 16
    hc = np.array([0, T], dtype=np.int32)
    hp = np.array([0], dtype=np.int32)
    ids = torch.zeros(T, dtype=torch.int32, device=G.DEV)
    batch, keep = cb.make_batch(ids, torch.from_numpy(hc).to(G.DEV), torch.from_numpy(hp).to(G.DEV), hc, hp)
    assert cb.confspec_static_scratch_need(ver.ctx, batch) > cb.STATIC_SCRATCH_BYTES
    table = torch.zeros((1, 1), dtype=torch.int32, device=G.DEV)
    pages = torch.zeros(16, dtype=torch.bfloat16, device=G.DEV)
    kv = cb.make_kv(pages, pages, table, 1, 16, 1)
    outs = ver.alloc_outputs(1, 2, 1)
    with pytest.raises(cb.ConfSpecError) as e:
        cb.confspec_verify_static(ver.ctx, ver.w, kv, batch, [1, 2], [0.9], *outs)
    assert e.value.code == cb.E_WORKSPACE and "static array" in str(e.value)
    ver.close()
