"""GPU parity of the pass with write-back (Algorithm 1, Stage 3) against the CPU oracle: the rows written into the
paged cache, that nothing else in the cache changes, that the verdict outputs are those of the plain pass, and that
a context built chunk by chunk by the GPU serves a later verification.

Bounds on the written keys / values (storage precision, relative to the largest magnitude of the reference rows of
the layer): bf16 2e-2 (the same drift through the layers that the 2e-2 bound on verdict logits allows, on values of
order one), fp32 1e-4."""
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
KV_TOL = {"bf16": 2e-2, "fp32": 1e-4}


def _rows(pages, table, b, lo, hi, bs):
    """Logical rows lo .. hi-1 of trace b from one layer's pages [n_blocks, Hkv, bs, hd] -> float64 [n, Hkv, hd]."""
    return np.stack([pages[int(table[b, j // bs]), :, j % bs, :].to(torch.float64).cpu().numpy() for j in range(lo, hi)])


def _check_appended(wl, batch, kv, before, n_app, ora, label):
    """Written rows against the oracle on ora['traces']; every other element of the cache unchanged."""
    m, bs = wl.model, wl.block_size
    table = batch.block_table.cpu().numpy()
    tol = KV_TOL[m.dtype]
    worst = 0.0
    for l in range(m.n_layers):
        for i, b in enumerate(ora["traces"]):
            L, n = int(batch.h_prefix_lens[b]), int(n_app[b])
            for name, pages, ref in (("k", kv.k_pages, ora["k"][l][i]), ("v", kv.v_pages, ora["v"][l][i])):
                if n == 0:
                    continue
                got = _rows(pages[l], table, b, L, L + n, bs)
                err = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-6)
                worst = max(worst, err)
                assert err <= tol, (label, name, l, b, err)
    # untouched: mask of written (block, slot) pairs, same for every layer and head
    written = torch.zeros(kv.k_pages.shape[1], bs, dtype=torch.bool)
    for b in range(wl.B):
        L = int(batch.h_prefix_lens[b])
        for j in range(L, L + int(n_app[b])):
            written[int(table[b, j // bs]), j % bs] = True
    keep = (~written).to(kv.k_pages.device)[None, :, None, :, None]
    for pages, old in ((kv.k_pages, before[0]), (kv.v_pages, before[1])):
        same = (pages.view(torch.int16 if pages.element_size() == 2 else torch.int32) ==
                old.view(torch.int16 if old.element_size() == 2 else torch.int32))
        assert bool((same | ~keep).all()), (label, "a row outside the appended ones changed")
    print(f"{label}: appended rows checked on traces {list(ora['traces'])}, worst relative error {worst:.2e}", flush=True)
    return worst


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_append_writes_oracle_rows_and_nothing_else(dtype):
    print(f"append {dtype}", flush=True)
    prefix = (0, 5, 77, 300, 16, 1000, 130)
    suffix = (1, 7, 33, 64, 100, 96, 250)
    n_app = np.array([1, 0, 33, 10, 17, 96, 129], dtype=np.int32)         # none, some, all; crossing block borders
    kw = dict(vocab=1024, block_size=16, prefix_lens=prefix, suffix_lens=suffix, taus=(0.5, 0.6))
    if dtype == "bf16":
        wl = W.tiny_workload("append", 5100, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2,
                             head_dim=128, d_ffn=768, **kw)
    else:
        wl = W.tiny_workload("append32", 5101, dtype="fp32", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4,
                             head_dim=64, d_ffn=512, **kw)
    weights = W.make_weights(wl.model, wl.seed, DEV)
    batch = W.make_batch(wl, DEV, extra_rows=n_app)
    kv = W.make_seeded_kv(wl, batch, DEV)
    before = (kv.k_pages.clone(), kv.v_pages.clone())
    vids = W.draw_verdict_ids(wl)
    ver = Verifier(wl.model, weights)
    plain = [t.clone() for t in ver.verify(kv, batch, vids, list(wl.taus))]
    torch.cuda.synchronize()
    ora = O.append_rows(wl.model, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                        batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, n_app)   # before the write
    outs = ver.verify_append(kv, batch, n_app, vids, list(wl.taus))
    torch.cuda.synchronize()
    for a, b in zip(plain, outs):
        assert torch.equal(a, b)                       # the write-back does not touch the verdict path
    _check_appended(wl, batch, kv, before, n_app, ora, f"append {dtype}")
    # argument checks: counts outside the suffix or past the block table
    for bad in (np.where(np.arange(7) == 2, 34, n_app), np.where(np.arange(7) == 1, -1, n_app)):
        with pytest.raises(cb.ConfSpecError) as e:
            ver.verify_append(kv, batch, bad.astype(np.int32), vids, list(wl.taus))
        assert e.value.code == cb.E_OUT_OF_RANGE
    tight = W.make_batch(wl, DEV)                       # block table without room for new rows
    with pytest.raises(cb.ConfSpecError) as e:
        ver.verify_append(kv, tight, n_app, vids, list(wl.taus))
    assert e.value.code == cb.E_OUT_OF_RANGE
    ver.close()


def test_context_built_chunk_by_chunk_on_the_gpu_serves_verification():
    """Chunked prefill from an empty cache (three passes with write-back of everything), then a plain verification
    on top of it: the cache against the oracle's single prefix pass, the verdicts against the oracle reading the
    cache the GPU wrote."""
    print("chunked prefill then verify", flush=True)
    total = (150, 37, 96, 211)                                          # context lengths to build
    wl0 = W.tiny_workload("chunks", 5200, dtype="bf16", n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2,
                          head_dim=128, d_ffn=768, vocab=1024, block_size=16, prefix_lens=total,
                          suffix_lens=(20, 9, 64, 33), taus=(0.5, 0.6))
    weights = W.make_weights(wl0.model, wl0.seed, DEV)
    final = W.make_batch(wl0, DEV)                                      # block table for the full contexts
    m = wl0.model
    ctx_ids = W.make_prefix_ids(wl0)
    dt = W.torch_dtype(m.dtype)
    shape = (m.n_layers, final.n_blocks, m.n_kv_heads, 16, m.head_dim)
    kv = W.KVCache(torch.zeros(shape, dtype=dt, device=DEV), torch.zeros(shape, dtype=dt, device=DEV), 16)
    ver = Verifier(m, weights)
    vids = W.draw_verdict_ids(wl0)
    done = np.zeros(4, dtype=np.int64)
    for frac in (0.4, 0.75, 1.0):
        upto = np.maximum(done + 1, np.round(np.asarray(total) * frac).astype(np.int64))
        upto = np.minimum(upto, total)
        chunk = [ctx_ids[b][done[b]:upto[b]] for b in range(4)]
        live = [b for b in range(4) if len(chunk[b])]
        cu = np.concatenate([[0], np.cumsum([len(chunk[b]) for b in live])]).astype(np.int32)
        part = W.Batch(suffix_ids=torch.from_numpy(np.concatenate([chunk[b] for b in live]).astype(np.int32)).to(DEV),
                       cu_suffix=torch.from_numpy(cu).to(DEV),
                       prefix_lens=torch.from_numpy(done[live].astype(np.int32)).to(DEV),
                       block_table=final.block_table[torch.as_tensor(live, device=DEV)].contiguous(),
                       n_blocks=final.n_blocks, max_blocks_per_seq=final.max_blocks_per_seq, block_size=16,
                       h_cu_suffix=cu, h_prefix_lens=done[live].astype(np.int32))
        ver.verify_append(kv, part, np.diff(cu), vids, [0.5])
        torch.cuda.synchronize()
        done = upto
    assert list(done) == list(total)
    k_ref, v_ref = O.prefix_pass(m, W.OracleModelView(weights), ctx_ids)
    table = final.block_table.cpu().numpy()
    worst = 0.0
    for l in range(m.n_layers):
        for b in range(4):
            for pages, ref in ((kv.k_pages, k_ref[l][b]), (kv.v_pages, v_ref[l][b])):
                got = _rows(pages[l], table, b, 0, total[b], 16)
                worst = max(worst, np.abs(got - ref).max() / np.abs(ref).max())
    print(f"cache built in chunks vs single prefix pass: worst relative error {worst:.2e}", flush=True)
    assert worst <= KV_TOL["bf16"]
    gpu = G.run_gpu(wl0, weights, final, kv, verifier=ver)
    ora = G.run_oracle(wl0, weights, final, kv, gpu["taus"], gpu["vids"])
    G.compare(wl0, gpu, ora, "verify on the GPU-built context")
    ver.close()


def test_append_full_size_config2_sampled_traces():
    print("append, config 2", flush=True)
    wl = W.config(2)
    n_app = np.full(wl.B, 40, dtype=np.int32)                          # a drafted step of 40 tokens joins every context
    n_app[5], n_app[31] = 0, 96
    weights = W.make_weights(wl.model, wl.seed, DEV)
    batch = W.make_batch(wl, DEV, extra_rows=n_app)
    kv = W.make_seeded_kv(wl, batch, DEV)
    before = (kv.k_pages.clone(), kv.v_pages.clone())
    vids = W.draw_verdict_ids(wl)
    ver = Verifier(wl.model, weights)
    plain = [t.clone() for t in ver.verify(kv, batch, vids, list(wl.taus))]
    torch.cuda.synchronize()
    sample = [0, 31]
    ora = O.append_rows(wl.model, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                        batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, n_app, trace_subset=sample)
    outs = ver.verify_append(kv, batch, n_app, vids, list(wl.taus))
    torch.cuda.synchronize()
    for a, b in zip(plain, outs):
        assert torch.equal(a, b)
    _check_appended(wl, batch, kv, before, n_app, ora, "append config 2")
    ver.close()


def test_full_size_context_built_by_chunked_prefill_then_verified():
    """Config 2's contexts (32 traces of 2048 tokens, 28 layers) built by this library's own kernels - four passes of
    512 context tokens per trace with write-back of everything - instead of seeded pages; then the verification
    pass on top, against the oracle reading the cache the GPU wrote, with the threshold sweep."""
    print("config 2 on a cache built by chunked prefill", flush=True)
    wl = W.config(2)
    m = wl.model
    weights = W.make_weights(m, wl.seed, DEV)
    final = W.make_batch(wl, DEV)
    ctx_ids = W.make_prefix_ids(wl)
    dt = W.torch_dtype(m.dtype)
    shape = (m.n_layers, final.n_blocks, m.n_kv_heads, 16, m.head_dim)
    kv = W.KVCache(torch.zeros(shape, dtype=dt, device=DEV), torch.zeros(shape, dtype=dt, device=DEV), 16)
    ver = Verifier(m, weights)
    vids = W.draw_verdict_ids(wl)
    chunk = 512
    for start in range(0, 2048, chunk):
        cu = (np.arange(wl.B + 1) * chunk).astype(np.int32)
        ids = np.concatenate([ctx_ids[b][start:start + chunk] for b in range(wl.B)]).astype(np.int32)
        done = np.full(wl.B, start, dtype=np.int32)
        part = W.Batch(suffix_ids=torch.from_numpy(ids).to(DEV), cu_suffix=torch.from_numpy(cu).to(DEV),
                       prefix_lens=torch.from_numpy(done).to(DEV), block_table=final.block_table,
                       n_blocks=final.n_blocks, max_blocks_per_seq=final.max_blocks_per_seq, block_size=16,
                       h_cu_suffix=cu, h_prefix_lens=done)
        ver.verify_append(kv, part, np.full(wl.B, chunk, dtype=np.int32), vids, [0.5])
        torch.cuda.synchronize()
    # one trace's context against the oracle's own prefix pass over the same tokens (keys / values of every layer)
    b = 17
    k_ref, v_ref = O.prefix_pass(m, W.OracleModelView(weights), [ctx_ids[b]])
    table = final.block_table.cpu().numpy()
    worst = 0.0
    for l in range(m.n_layers):
        for pages, ref in ((kv.k_pages, k_ref[l][0]), (kv.v_pages, v_ref[l][0])):
            got = _rows(pages[l], table, b, 0, 2048, 16)
            worst = max(worst, np.abs(got - ref).max() / np.abs(ref).max())
    print(f"trace {b}: context built in chunks vs the oracle's prefix pass, worst relative error {worst:.2e}", flush=True)
    assert worst <= KV_TOL["bf16"]
    taus = G.sweep_taus(wl)
    gpu = G.run_gpu(wl, weights, final, kv, taus=taus, verifier=ver)
    ora = G.run_oracle(wl, weights, final, kv, gpu["taus"], gpu["vids"], traces=[3, 17, 28])
    s = G.compare(wl, gpu, ora, "config 2 on the GPU-built context")
    assert s["gate_kept"] > 0 and s["gate_escalated"] > 0, s
    ver.close()


def test_append_of_nothing_leaves_the_cache_alone():
    print("append nothing", flush=True)
    wl = W.tiny_workload("append0", 5300, dtype="bf16", n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128,
                         d_ffn=768, vocab=1024, block_size=16, prefix_lens=(33, 0, 160), suffix_lens=(5, 1, 40), taus=(0.5,))
    weights = W.make_weights(wl.model, wl.seed, DEV)
    batch = W.make_batch(wl, DEV)
    kv = W.make_seeded_kv(wl, batch, DEV)
    before = (kv.k_pages.clone(), kv.v_pages.clone())
    ver = Verifier(wl.model, weights)
    vids = W.draw_verdict_ids(wl)
    plain = [t.clone() for t in ver.verify(kv, batch, vids, [0.5])]
    outs = ver.verify_append(kv, batch, np.zeros(3, dtype=np.int32), vids, [0.5])
    torch.cuda.synchronize()
    assert torch.equal(kv.k_pages, before[0]) and torch.equal(kv.v_pages, before[1])
    for a, b in zip(plain, outs):
        assert torch.equal(a, b)
    ver.close()
