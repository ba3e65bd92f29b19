#!/usr/bin/env python3
"""Benchmark of the batched verification pass on one MI355X.

One step = one confspec_verify call (every kernel of the pass) over one synthetic batch that is
already resident in HBM.  Prints one JSON line: verified steps/s, the MFMA roofline of the dominant
kernel (the gate/up projection GEMM with its SwiGLU epilogue) measured live with HIP events, and the
CPU oracle timed on a bounded sample of the same workload as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
GEMM_SOURCE = os.path.join(ROOT, "paper_2602_18447_amd", "csrc", "gemm_bf16.hip")
HBM_COUNTERS = os.path.join(ROOT, "profiles", "gate_up_gemm_config2_hbm_counters.json")


def _hbm_traffic():
    """HBM bytes per launch of the gate/up GEMM from the stored hardware-counter runs, or None when
    there is no record or the kernel source has changed since the counters were taken."""
    import hashlib

    try:
        with open(HBM_COUNTERS) as f:
            rec = json.load(f)
        with open(GEMM_SOURCE, "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()
    except OSError:
        return None
    if rec.get("gemm_source_sha256") != sha:
        return None
    return rec.get("gate_up_gemm")


def _blas_threads():
    """Threads the oracle's BLAS calls run on (numpy's pool), not the machine's core count."""
    try:
        from threadpoolctl import threadpool_info

        n = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    return os.cpu_count()


def _time_cascade(W, wl, draft_ver, draft_kv, batch, vids, dev, reps):
    """Wall time of confspec_cascade calls (they synchronise once inside, so host time is the measure): the small
    model's pass over every trace, selection, and the large model's pass over the escalated sub-batch.  Requests of
    1 to 5 drafted steps."""
    import numpy as np
    import torch

    from paper_2602_18447_amd.runner import Cascade, Verifier

    wl_t = W.Workload("cascade_target", W.TARGET_SHAPE, wl.seed + 10, wl.prefix_lens, wl.suffix_lens)
    w_t = W.make_weights(wl_t.model, wl_t.seed, dev)
    kv_t = W.make_seeded_kv(wl_t, batch, dev)
    tgt = Verifier(wl_t.model, w_t)
    casc = Cascade(draft_ver, tgt)
    req = [0]
    k = 1
    while req[-1] < wl.B:
        req.append(min(req[-1] + k, wl.B))
        k = k % 5 + 1
    outs = casc.alloc_outputs(wl.B, len(req) - 1)
    res = {}
    for gamma in (0.9, 0.6):
        for _ in range(2):
            _, n_t = casc.run(draft_kv, kv_t, batch, req, vids, gamma, outputs=outs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            casc.run(draft_kv, kv_t, batch, req, vids, gamma, outputs=outs)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        res[f"gamma_{gamma}"] = dict(ms_per_call=round(ms, 3), traces_in_large_pass=n_t,
                                     escalated=int(outs["escalated"].sum().item()),
                                     accepted_steps=int(outs["accepted_steps"].sum().item()),
                                     steps_decided_per_s=round(wl.B / (ms * 1e-3), 1))
    # the large model alone on the whole batch, for scale
    o_t = tgt.alloc_outputs(wl.B, len(vids), 1)
    for _ in range(2):
        tgt.verify(kv_t, batch, vids, [0.9], outputs=o_t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        tgt.verify(kv_t, batch, vids, [0.9], outputs=o_t)
    torch.cuda.synchronize()
    res["large_model_whole_batch_ms"] = round((time.perf_counter() - t0) / reps * 1e3, 3)
    res["requests"] = len(req) - 1
    res["large_model"] = dict(layers=wl_t.model.n_layers, d_model=wl_t.model.d_model)
    tgt.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload: 2 (default, the metric's config), 3, 4 or 5")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP-graph replays")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="confspec_tune setting applied before the run (repeatable), for measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the plain copy kernel (1 GiB, 5 times): the yardstick for HBM byte counters")
    ap.add_argument("--cascade", action="store_true",
                    help="also time the two-tier cascade call (this workload's batch, the 32B-shaped model as the large "
                         "one, gamma 0.9 and 0.6) and report it under \"cascade\"")
    ap.add_argument("--append", type=int, default=0, metavar="N",
                    help="also time the pass with write-back of the first N suffix tokens of every trace into the "
                         "cache and report it under \"append\"")
    ap.add_argument("--shared-prefix", type=int, default=0, metavar="W",
                    help="also time the pass with groups of W traces reading the same context pages (the W candidates of "
                         "one step in tree-structured drafting) and report it under \"shared_prefix\"")
    ap.add_argument("--decode", type=int, default=0, metavar="N",
                    help="also time N greedy generation steps (one new token per trace, keys / values appended, "
                         "full-vocabulary head) on this workload's contexts and report them under \"decode\"")
    ap.add_argument("--cpu-baseline-traces", type=int, default=6,
                    help="traces of the workload the CPU oracle is timed on (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (traces are independent; more GPUs would each take a "
              "share of the traces with a replica of the weights, no collectives) - rerun with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import confspec_workloads as W
    from paper_2602_18447_amd import binding as cb
    from paper_2602_18447_amd.runner import Verifier

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    for kv_ in args.tune:
        key, _, val = kv_.partition("=")
        cb.confspec_tune(None, key, int(val))      # defaults of the contexts created below
    wl = W.config(args.config)
    m = wl.model
    weights = W.make_weights(m, wl.seed, dev)
    batch = W.make_batch(wl, dev)
    kv = W.make_seeded_kv(wl, batch, dev)
    vids = W.draw_verdict_ids(wl)
    taus = list(wl.taus)
    ver = Verifier(m, weights)
    outs = ver.alloc_outputs(wl.B, len(vids), len(taus))
    ver.workspace(wl.T, wl.B)
    torch.cuda.synchronize()

    # Eager launches first (also the reference result for the graph replays below).
    for _ in range(max(args.warmup, 1)):
        ver.verify(kv, batch, vids, taus, outputs=outs)
    torch.cuda.synchronize()
    eager_logits = outs[0].clone()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        ver.verify(kv, batch, vids, taus, outputs=outs)
    e1.record()
    torch.cuda.synchronize()
    eager_ms = e0.elapsed_time(e1) / args.steps

    # The call allocates nothing and never synchronises, so it can be captured once into a HIP graph and
    # replayed: one step = one replay of the whole pass (every kernel of confspec_verify).
    graph_ok = not args.no_graph
    if graph_ok:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ver.verify(kv, batch, vids, taus, outputs=outs)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ver.verify(kv, batch, vids, taus, outputs=outs)
        for i in range(max(args.warmup, 2)):           # replays checked against the eager result
            outs[0].zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not torch.equal(outs[0], eager_logits):
                graph_ok = False
                break
    if graph_ok:
        e0.record()
        for _ in range(args.steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ms_per_step = e0.elapsed_time(e1) / args.steps
    else:
        ms_per_step = eager_ms
    steps_per_s = wl.B / (ms_per_step * 1e-3)
    accept_counts = outs[3].cpu().numpy().sum(axis=1).tolist()

    # ---- roofline of the dominant operation: gate/up GEMM + SwiGLU (two launches back to back), same shape and
    # launch configuration as in the pass; time per projection = sum of the two kernels
    T, d, F = wl.T, m.d_model, m.d_ffn
    h = (torch.randn(T, d, device=dev) * 0.5).to(torch.bfloat16)
    act = torch.empty(T, F, dtype=torch.bfloat16, device=dev)
    packed_ptrs = ver._packed_ptrs

    class _Raw:   # pointer of one layer's packed gate/up matrix
        def __init__(self, p):
            self.p = p

        def data_ptr(self):
            return self.p

    n_launch = max(args.steps, 1) * m.n_layers
    for l in range(m.n_layers):
        cb.confspec_op_gemm(ver.ctx, h, _Raw(packed_ptrs[l]), act, T, 2 * F, d, cb.EPI_SWIGLU)
    torch.cuda.synchronize()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record()
    for i in range(n_launch):
        cb.confspec_op_gemm(ver.ctx, h, _Raw(packed_ptrs[i % m.n_layers]), act, T, 2 * F, d, cb.EPI_SWIGLU)
    g1.record()
    torch.cuda.synchronize()
    gemm_ms = g0.elapsed_time(g1) / n_launch
    gemm_flops = 2.0 * T * (2 * F) * d
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
    traffic = _hbm_traffic() if args.config == 2 else None   # the counters were taken on config 2's shape
    roofline = dict(bound="mfma",
                    kernel="gate/up projection + SwiGLU of a bf16 layer: gemm_bf16_kernel<256,256,2,4,64,2,2,1> on the "
                           "columns that fill whole rounds of 256 tiles + gemm_bf16_kernel<128,128,2,2,64,2,2,1> on the rest",
                    achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                    traffic=None if traffic is None else traffic["hbm_bytes"],
                    traffic_detail=traffic, flops_per_launch=gemm_flops,
                    algorithmic_bytes_per_launch=2 * (T * d + 2 * F * d + T * F),
                    avg_launch_ms=round(gemm_ms, 5), launches_timed=n_launch)

    copy_info = None
    if args.calibrate_copy:
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        cb.confspec_op_copy(src, dst, nbytes)
        torch.cuda.synchronize()
        g0.record()
        for _ in range(5):
            cb.confspec_op_copy(src, dst, nbytes)
        g1.record()
        torch.cuda.synchronize()
        copy_ms = g0.elapsed_time(g1) / 5
        if not torch.equal(src, dst):
            raise RuntimeError("copy kernel result differs from its source")
        copy_info = dict(bytes_read=nbytes, bytes_written=nbytes, avg_ms=round(copy_ms, 4),
                         GBps=round(2 * nbytes / (copy_ms * 1e-3) / 1e9, 1))
        del src, dst

    append_info = None
    if args.append > 0:
        n_app = np.minimum(np.asarray(wl.suffix_lens), args.append).astype(np.int32)
        batch_a = W.make_batch(wl, dev, extra_rows=n_app)           # same ids and blocks, a block table with room
        kv_a = W.make_seeded_kv(wl, batch_a, dev)
        for _ in range(3):
            ver.verify_append(kv_a, batch_a, n_app, vids, taus, outputs=outs)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            ver.verify_append(kv_a, batch_a, n_app, vids, taus, outputs=outs)
        e1.record()
        torch.cuda.synchronize()
        ms_a = e0.elapsed_time(e1) / args.steps
        rows = int(n_app.sum())
        append_info = dict(ms_per_step=round(ms_a, 4), launch="eager", tokens_appended=rows,
                           bytes_written=rows * m.n_layers * 2 * m.n_kv_heads * m.head_dim * (2 if m.dtype == "bf16" else 4),
                           extra_ms_vs_eager_pass=round(ms_a - eager_ms, 4))

    shared_info = None
    if args.shared_prefix > 1:
        import copy
        Wd = args.shared_prefix
        batch_s = copy.copy(batch)
        table = batch.block_table.clone()
        for b in range(wl.B):
            table[b] = batch.block_table[b - b % Wd]         # prefix lengths are equal inside a group in this workload
        batch_s.block_table = table
        for _ in range(3):
            ver.verify(kv, batch_s, vids, taus, outputs=outs)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            ver.verify(kv, batch_s, vids, taus, outputs=outs)
        e1.record()
        torch.cuda.synchronize()
        ms_s = e0.elapsed_time(e1) / args.steps
        shared_info = dict(group=Wd, ms_per_step=round(ms_s, 4), launch="eager", distinct_pages_ms_per_step=round(eager_ms, 4),
                           context_bytes_distinct=int(sum(wl.prefix_lens)) * m.n_layers * 2 * m.n_kv_heads * m.head_dim * 2,
                           context_bytes_shared=int(sum(wl.prefix_lens[::Wd])) * m.n_layers * 2 * m.n_kv_heads * m.head_dim * 2)

    decode_info = None
    if args.decode > 0:
        nst = args.decode
        batch_d = W.make_batch(wl, dev, extra_rows=2 * nst)
        kv_d = W.make_seeded_kv(wl, batch_d, dev)
        first = batch_d.suffix_ids[batch_d.cu_suffix[:-1].long()].contiguous()      # one starting token per trace
        L0 = batch_d.h_prefix_lens
        ver.generate_greedy(kv_d, batch_d.block_table, batch_d.n_blocks, batch_d.max_blocks_per_seq, first, L0, nst)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        toks, _, _ = ver.generate_greedy(kv_d, batch_d.block_table, batch_d.n_blocks, batch_d.max_blocks_per_seq, first,
                                         L0 + nst, nst)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        wbytes = sum(t.numel() * t.element_size() for l in range(m.n_layers)
                     for t in (weights.wqkv[l], weights.wo[l], weights.w_gate_up[l], weights.w_down[l]))
        wbytes += weights.lm_head.numel() * weights.lm_head.element_size()
        kvbytes = int(sum(wl.prefix_lens)) * m.n_layers * 2 * m.n_kv_heads * m.head_dim * weights.lm_head.element_size()
        decode_info = dict(steps=nst, ms_per_step=round(dt / nst * 1e3, 4), tokens_per_s=round(wl.B * nst / dt, 1),
                           launch="eager", algorithmic_bytes_per_step=wbytes + kvbytes,
                           achieved_TBps=round((wbytes + kvbytes) / (dt / nst) / 1e12, 3))
        # the same step without the host's launch work: one step (fixed context lengths) captured into a HIP graph and
        # replayed; the replays rewrite the same cache rows with the same values
        from types import SimpleNamespace
        cu1 = np.arange(wl.B + 1, dtype=np.int32)
        one = SimpleNamespace(suffix_ids=first, cu_suffix=torch.from_numpy(cu1).to(dev), prefix_lens=batch_d.prefix_lens,
                              block_table=batch_d.block_table, n_blocks=batch_d.n_blocks,
                              max_blocks_per_seq=batch_d.max_blocks_per_seq, block_size=kv_d.block_size,
                              h_cu_suffix=cu1, h_prefix_lens=L0)
        ones = np.ones(wl.B, dtype=np.int32)
        ones_dev = torch.from_numpy(ones).to(dev)
        g_out = ver.generate_step(kv_d, one, n_append=ones, n_append_dev=ones_dev)
        torch.cuda.synchronize()
        ref_tok = g_out["token"].clone()
        side2 = torch.cuda.Stream()
        side2.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side2):
            ver.generate_step(kv_d, one, n_append=ones, n_append_dev=ones_dev, outputs=g_out)
        torch.cuda.current_stream().wait_stream(side2)
        torch.cuda.synchronize()
        dgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(dgraph):
            ver.generate_step(kv_d, one, n_append=ones, n_append_dev=ones_dev, outputs=g_out)
        ok = True
        for _ in range(3):
            g_out["token"].zero_()
            dgraph.replay()
            torch.cuda.synchronize()
            ok = ok and torch.equal(g_out["token"], ref_tok)
        if ok:
            e0.record()
            for _ in range(nst):
                dgraph.replay()
            e1.record()
            torch.cuda.synchronize()
            ms_g = e0.elapsed_time(e1) / nst
            decode_info.update(graph_ms_per_step=round(ms_g, 4), graph_tokens_per_s=round(wl.B / (ms_g * 1e-3), 1),
                               graph_achieved_TBps=round((wbytes + kvbytes) / (ms_g * 1e-3) / 1e12, 3))

    cascade_info = None
    if args.cascade:
        cascade_info = _time_cascade(W, wl, ver, kv, batch, vids, dev, max(args.steps // 2, 3))

    # ---- CPU oracle on a bounded sample of the same workload (reported baseline only)
    cpu = None
    if args.cpu_baseline_traces > 0:
        from oracle import confspec_oracle as O

        n = min(args.cpu_baseline_traces, wl.B)
        t0 = time.time()
        ora = O.verify(m, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                       batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, vids, taus,
                       trace_subset=list(range(n)))
        dt = time.time() - t0
        # eager_logits: the timed pass's own output (the optional legs above reuse the output buffers)
        dl = float(np.abs(eager_logits.cpu().numpy()[:n] - ora["logits"]).max())
        cpu = dict(value=round(n / dt, 4), unit="verified steps/s", cores=_blas_threads(), kind="oracle",
                   sample=f"first {n} of {wl.B} traces of {wl.name}, fp64 numpy, {dt:.1f} s",
                   max_abs_dlogit_vs_gpu=dl)

    print(json.dumps({
        "metric": "verified steps/sec (batched verify pass)", "value": round(steps_per_s, 1),
        "unit": "verified steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "T": wl.T, "sum_prefix_len": int(sum(wl.prefix_lens)),
                   "layers": m.n_layers, "d_model": m.d_model, "taus": taus, "accept_counts": accept_counts,
                   "launch": "hip_graph_replay" if graph_ok else "eager", "eager_ms_per_step": round(eager_ms, 4),
                   **({"tune": args.tune} if args.tune else {})},
        "roofline": roofline, "cpu_baseline": cpu, **({"copy_calibration": copy_info} if copy_info else {}),
        **({"cascade": cascade_info} if cascade_info else {}), **({"append": append_info} if append_info else {}),
        **({"shared_prefix": shared_info} if shared_info else {}), **({"decode": decode_info} if decode_info else {}),
    }))


if __name__ == "__main__":
    main()
