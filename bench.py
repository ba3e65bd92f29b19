#!/usr/bin/env python3
"""Benchmark of the batched verification pass on one MI355X.

One step = one confspec_verify call (every kernel of the pass) over one synthetic batch that is already
resident in HBM, replayed as a HIP graph.  The default run times the four bf16 workloads (configs 2-5) one
after the other and prints ONE JSON line: the headline figures are those of the largest single-GPU workload
(config 4, the ragged 128-trace batch); `per_config` carries every workload's pass time, the executed-flop
rate of each projection and of attention taken from HIP events inside the pass, and the CPU oracle timed on
a bounded sample of the same workload.  `--config N` runs one workload only (and makes it the headline).
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 MFMA
PEAK_HBM_GBPS = 8000.0
CSRC = os.path.join(ROOT, "paper_2602_18447_amd", "csrc")
HEADLINE_CONFIG = 4
# traces of each workload the CPU oracle is timed on by default: about 10-20 s of CPU work for the headline
# workload, a few seconds for the others
CPU_SAMPLE = {2: 3, 3: 2, 4: 6, 5: 1}
# thresholds added to each workload's own so that both gate outcomes occur at random-init confidences
EXTRA_TAUS = (0.55, 0.6, 0.7)


def _counter_record(name, sources):
    """Stored hardware-counter record profiles/<name>, or None when there is none or a kernel source it was taken
    on has changed since."""
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            rec = json.load(f)
        h = hashlib.sha256()
        for src in sources:
            with open(os.path.join(CSRC, src), "rb") as f:
                h.update(f.read())
    except (OSError, ValueError):
        return None
    return rec if rec.get("source_sha256") == h.hexdigest() else None


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


def _work(wl, n_f16_layers):
    """Executed work of one pass by phase (flops; context bytes for attention).  The last layer runs its
    attention rows, output projection and MLP on the last position of each trace only."""
    m = wl.model
    T, B, n = wl.T, wl.B, m.n_layers
    qw, kw = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    L = [int(v) for v in wl.prefix_lens]
    S = [int(v) for v in wl.suffix_lens]
    per_row_key = 4.0 * m.head_dim                       # QK^T and PV, per q head, query row and visible key
    attn_full = sum(m.n_q_heads * s * (l + (s + 1) / 2.0) for l, s in zip(L, S)) * per_row_key
    attn_last = sum(m.n_q_heads * (l + s) for l, s in zip(L, S)) * per_row_key
    kv_layer = sum(L) * 2 * kw * 2                        # context keys + values of one layer, bytes
    rows = (n - 1) * T + B                                # rows the residual projections and the MLP run on
    return dict(
        qkv=2.0 * n * T * (qw + 2 * kw) * m.d_model,
        o_proj=2.0 * rows * m.d_model * qw,
        gate_up=2.0 * rows * 2 * m.d_ffn * m.d_model,
        down=2.0 * rows * m.d_model * m.d_ffn,
        attn=(n - 2) * attn_full + attn_last if n >= 2 else 0.0,      # layers 1 .. n-1 (one-term kernel)
        attn_precise=attn_full if n >= 2 else attn_last,               # layer 0 (two-term kernel)
        attn_layer=attn_full, kv_layer_bytes=kv_layer,
        formats=dict(fp16_layers=n_f16_layers, bf16_layers=n - n_f16_layers),
    )


def _run_config(cfg_id, args, dev, cpu_traces):
    import numpy as np
    import torch

    import confspec_workloads as W
    from paper_2602_18447_amd import binding as cb
    from paper_2602_18447_amd.runner import Verifier

    wl = W.config(cfg_id)
    m = wl.model
    t_in = time.time()
    weights = W.make_weights(m, wl.seed, dev)
    batch = W.make_batch(wl, dev)
    kv = W.make_seeded_kv(wl, batch, dev)
    vids = W.draw_verdict_ids(wl)
    taus = sorted(set(float(t) for t in wl.taus) | set(EXTRA_TAUS))
    ver = Verifier(m, weights)
    outs = ver.alloc_outputs(wl.B, len(vids), len(taus))
    ver.workspace(wl.T, wl.B)
    torch.cuda.synchronize()
    t_in = time.time() - t_in

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

    # Phase times from HIP events recorded inside the pass, on the pass's stream (eager launches).
    cb.confspec_phase_timing(ver.ctx, True)
    n_timed = max(2, min(args.steps, 5))
    acc = {}
    for _ in range(n_timed):
        ver.verify(kv, batch, vids, taus, outputs=outs)
        for k, (ms, cnt) in cb.confspec_phase_times(ver.ctx).items():
            a = acc.setdefault(k, [0.0, 0])
            a[0] += ms / n_timed
            a[1] = cnt
    cb.confspec_phase_timing(ver.ctx, False)

    # The call allocates nothing and never synchronises, so it is captured once into a HIP graph and replayed:
    # one step = one replay of the whole pass.
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
        for i in range(max(min(args.warmup, 3), 2)):           # replays checked against the eager result
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
    accept_counts = outs[3].cpu().numpy().sum(axis=1).tolist()
    conf = outs[1].cpu().numpy()

    wk = _work(wl, ver.w.n_f16_layers)
    tf = lambda flops, ms: flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0   # noqa: E731
    gemms = {}
    for k in ("qkv", "o_proj", "gate_up", "down"):
        ms = acc[k][0]
        r = tf(wk[k], ms)
        gemms[k] = dict(ms_per_pass=round(ms, 4), executed_gflop=round(wk[k] / 1e9, 1), tflops=round(r, 1),
                        frac_of_peak=round(r / PEAK_BF16_TFLOPS, 4))
    g_ms = sum(acc[k][0] for k in gemms)
    g_fl = sum(wk[k] for k in gemms)
    gemms["all"] = dict(ms_per_pass=round(g_ms, 4), executed_gflop=round(g_fl / 1e9, 1), tflops=round(tf(g_fl, g_ms), 1),
                        frac_of_peak=round(tf(g_fl, g_ms) / PEAK_BF16_TFLOPS, 4),
                        note="down includes its split-K reduce / residual / next-RMSNorm kernel where the projection is cut in k")
    a_ms, a_cnt = acc["attn"]
    attn = dict(kernel_ms_per_pass=round(a_ms, 4), launches=a_cnt, avg_launch_ms=round(a_ms / max(a_cnt, 1), 5),
                executed_gflop=round(wk["attn"] / 1e9, 1), tflops=round(tf(wk["attn"], a_ms), 1),
                frac_of_peak=round(tf(wk["attn"], a_ms) / PEAK_BF16_TFLOPS, 4),
                context_GBps=round(wk["kv_layer_bytes"] * a_cnt / (a_ms * 1e-3) / 1e9, 1) if a_ms > 0 else None,
                merge_ms_per_pass=round(acc["attn_merge"][0], 4),
                two_term_first_layer_ms=round(acc["attn_precise"][0], 4))
    phases = {k: round(v[0], 4) for k, v in acc.items()}

    cpu = None
    if cpu_traces > 0:
        from oracle import confspec_oracle as O

        n = min(cpu_traces, wl.B)
        t0 = time.time()
        ora = O.verify(m, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                       batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, vids, taus,
                       trace_subset=list(range(n)))
        dt = time.time() - t0
        dl = float(np.abs(eager_logits.cpu().numpy()[:n] - ora["logits"]).max())
        cpu = dict(value=round(n / dt, 4), unit="verified steps/s", cores=_blas_threads(), kind="oracle",
                   sample=f"first {n} of {wl.B} traces of {wl.name}, fp64 numpy, {dt:.1f} s",
                   max_abs_dlogit_vs_gpu=dl)

    entry = dict(workload=wl.name, config=cfg_id, B=wl.B, T=wl.T, sum_prefix_len=int(sum(wl.prefix_lens)),
                 ms_per_step=round(ms_per_step, 4), verified_steps_per_s=round(wl.B / (ms_per_step * 1e-3), 1),
                 launch="hip_graph_replay" if graph_ok else "eager", eager_ms_per_step=round(eager_ms, 4),
                 taus=taus, accept_counts=accept_counts, conf_min_max=[round(float(conf.min()), 4), round(float(conf.max()), 4)],
                 gemm=gemms, operand_formats=wk["formats"], attention=attn, phase_ms_per_pass=phases,
                 input_setup_s=round(t_in, 1), cpu_baseline=cpu)
    state = dict(wl=wl, weights=weights, batch=batch, kv=kv, vids=vids, taus=taus, ver=ver, outs=outs, eager_ms=eager_ms,
                 acc=acc, work=wk, passes_timed=n_timed)
    return entry, state


def _roofline(entry, state):
    """Roofline of the kernel the pass spends most of its time in: attention or the gate/up projection."""
    acc, wk, wl = state["acc"], state["work"], state["wl"]
    m = wl.model
    label = "bytes that missed L2 (FETCH_SIZE + WRITE_SIZE): served by HBM or the 256 MB last-level cache"
    if acc["attn"][0] >= acc["gate_up"][0]:
        ms, cnt = acc["attn"]
        achieved = wk["attn"] / (ms * 1e-3) / 1e12
        rec = _counter_record(f"attention_config{entry['config']}_l2_miss_counters.json", ["attn_bf16.hip"])
        return dict(bound="mfma",
                    kernel="attention over paged context + suffix (one-term kernel; one launch per layer from the second "
                           "layer on, the last one on the last position of each trace only)",
                    achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                    traffic=None if rec is None else rec["l2_miss_bytes_per_launch"], traffic_label=label,
                    traffic_detail=rec, flops_per_launch=wk["attn"] / max(cnt, 1),
                    algorithmic_bytes_per_launch=wk["kv_layer_bytes"],
                    avg_launch_ms=round(ms / max(cnt, 1), 5), launches_timed=cnt * state["passes_timed"],
                    context_stream_GBps=entry["attention"]["context_GBps"], hbm_peak_GBps=PEAK_HBM_GBPS)
    ms, cnt = acc["gate_up"]
    achieved = wk["gate_up"] / (ms * 1e-3) / 1e12
    T, d, F = wl.T, m.d_model, m.d_ffn
    rec = _counter_record(f"gate_up_gemm_config{entry['config']}_l2_miss_counters.json", ["gemm_bf16.hip"])
    return dict(bound="mfma", kernel="gate/up projection + SwiGLU (256x256 tiles, trailing columns on 128x128 tiles)",
                achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                traffic=None if rec is None else rec["l2_miss_bytes_per_launch"], traffic_label=label,
                traffic_detail=rec, flops_per_launch=wk["gate_up"] / max(cnt, 1),
                algorithmic_bytes_per_launch=2 * (T * d + 2 * F * d + T * F),
                avg_launch_ms=round(ms / max(cnt, 1), 5), launches_timed=cnt * state["passes_timed"])


def _time_cascade(W, wl, draft_ver, draft_kv, batch, vids, dev, reps):
    """Wall time of confspec_cascade calls (they synchronise once inside, so host time is the measure): the small
    model's pass over every trace, selection, and the large model's pass over the escalated sub-batch.  Requests of
    1 to 5 drafted steps."""
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


def _optional_legs(args, st, dev):
    """Extra measurements on one workload (only with --config N)."""
    import numpy as np
    import torch

    import confspec_workloads as W

    wl, weights, batch, kv, vids, taus, ver, outs = (st[k] for k in ("wl", "weights", "batch", "kv", "vids", "taus", "ver", "outs"))
    m = wl.model
    eager_ms = st["eager_ms"]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    extra = {}

    if args.calibrate_copy:
        # a plain streaming kernel of known size - every byte of a 1 GiB buffer read once, its complement written to a
        # second one (torch's element-wise kernel for bitwise_not, a name nothing else in the run uses): the yardstick
        # that the FETCH_SIZE / WRITE_SIZE counters of the other kernels are scaled by
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        torch.bitwise_not(src, out=dst)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            torch.bitwise_not(src, out=dst)
        e1.record()
        torch.cuda.synchronize()
        copy_ms = e0.elapsed_time(e1) / 5
        extra["copy_calibration"] = dict(kernel="bitwise_not", bytes_read=nbytes, bytes_written=nbytes, launches=6,
                                         avg_ms=round(copy_ms, 4), GBps=round(2 * nbytes / (copy_ms * 1e-3) / 1e9, 1))
        del src, dst

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
        extra["append"] = dict(ms_per_step=round(ms_a, 4), launch="eager", tokens_appended=rows,
                               bytes_written=rows * m.n_layers * 2 * m.n_kv_heads * m.head_dim * 2,
                               extra_ms_vs_eager_pass=round(ms_a - eager_ms, 4))

    if args.shared_prefix > 1:
        # Groups of W traces as the W candidates of one step (Section 4.3): their block-table rows name the same pages.
        # "aliased": the plain pass on that batch (pages shared, every candidate tiled on its own);
        # "grouped": confspec_verify_shared (the candidates of a group side by side in the attention row tiles).
        # Measured for the workload's own suffix lengths and for short steps of 16 tokens.
        import copy
        Wd = args.shared_prefix
        gstart = list(range(0, wl.B, Wd)) + [wl.B]
        G_, Hkv = m.n_q_heads // m.n_kv_heads, m.n_kv_heads

        def stagings(S, L, groups):
            tiles = lambda rows: -(-rows // 128)   # noqa: E731
            plain = sum(Hkv * tiles(G_ * s_) * -(-l_ // 64) for s_, l_ in zip(S, L))
            grouped = sum(Hkv * tiles(G_ * sum(S[lo:hi])) * -(-L[lo] // 64) for lo, hi in zip(groups[:-1], groups[1:]))
            return plain, grouped

        def timed(fn):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        res = {}
        for label, wl_s in (("own_suffix", wl), ("suffix_16", W.Workload(wl.name + "_s16", m, wl.seed, wl.prefix_lens, (16,) * wl.B))):
            b_s = batch if wl_s is wl else W.make_batch(wl_s, dev)
            kv_s = kv if wl_s is wl else W.make_seeded_kv(wl_s, b_s, dev)
            b_s = copy.copy(b_s)
            table = b_s.block_table.clone()
            for b in range(wl.B):
                table[b] = b_s.block_table[b - b % Wd]         # prefix lengths are equal inside a group in these workloads
            b_s.block_table = table
            o_s = ver.alloc_outputs(wl.B, len(vids), len(taus))
            ms_alias = timed(lambda: ver.verify(kv_s, b_s, vids, taus, outputs=o_s))
            ref = o_s[0].clone()
            ms_group = timed(lambda: ver.verify_shared(kv_s, b_s, gstart, vids, taus, outputs=o_s))
            torch.cuda.synchronize()
            plain_st, grouped_st = stagings(list(wl_s.suffix_lens), list(wl_s.prefix_lens), gstart)
            res[label] = dict(aliased_ms_per_step=round(ms_alias, 4), grouped_ms_per_step=round(ms_group, 4),
                              context_chunk_stagings_per_layer=dict(aliased=plain_st, grouped=grouped_st),
                              max_abs_dlogit_grouped_vs_aliased=float((o_s[0] - ref).abs().max().item()))
        extra["shared_prefix"] = dict(group=Wd, launch="eager", distinct_pages_ms_per_step=round(eager_ms, 4), **res)

    if args.decode > 0:
        nst = args.decode
        batch_d = W.make_batch(wl, dev, extra_rows=2 * nst)
        kv_d = W.make_seeded_kv(wl, batch_d, dev)
        first = batch_d.suffix_ids[batch_d.cu_suffix[:-1].long()].contiguous()      # one starting token per trace
        L0 = batch_d.h_prefix_lens
        ver.generate_greedy(kv_d, batch_d.block_table, batch_d.n_blocks, batch_d.max_blocks_per_seq, first, L0, nst)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ver.generate_greedy(kv_d, batch_d.block_table, batch_d.n_blocks, batch_d.max_blocks_per_seq, first, L0 + nst, nst)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        wbytes = sum(t.numel() * t.element_size() for l in range(m.n_layers)
                     for t in (weights.wqkv[l], weights.wo[l], weights.w_gate_up[l], weights.w_down[l]))
        wbytes += weights.lm_head.numel() * weights.lm_head.element_size()
        kvbytes = int(sum(wl.prefix_lens)) * m.n_layers * 2 * m.n_kv_heads * m.head_dim * weights.lm_head.element_size()
        info = dict(steps=nst, ms_per_step=round(dt / nst * 1e3, 4), tokens_per_s=round(wl.B * nst / dt, 1),
                    launch="eager", algorithmic_bytes_per_step=wbytes + kvbytes,
                    achieved_TBps=round((wbytes + kvbytes) / (dt / nst) / 1e12, 3),
                    # the step's own kernels (one token per trace, B <= 32, d_model <= 1536): per layer QKV + rotation + cache write,
                    # attention, output projection, gate/up + SwiGLU, down projection; around them position / rotary
                    # tables, embedding, counters, first RMSNorm, final RMSNorm, head with running arg max /
                    # log-sum-exp, its last reduction
                    kernel_launches_per_step=(5 * m.n_layers + 8 if wl.B <= 32 and m.d_model <= 1536 and
                                              m.n_q_heads * m.head_dim <= 1536 and "decode_kernels=0" not in args.tune
                                              else None))
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
            info.update(graph_ms_per_step=round(ms_g, 4), graph_tokens_per_s=round(wl.B / (ms_g * 1e-3), 1),
                        graph_achieved_TBps=round((wbytes + kvbytes) / (ms_g * 1e-3) / 1e12, 3))
        extra["decode"] = info

    if args.cascade:
        extra["cascade"] = _time_cascade(W, wl, ver, kv, batch, vids, dev, max(args.steps // 2, 3))

    if args.vendor_gemm:
        # Context, not a target: the vendor BLAS library (through torch.matmul, bf16, no fused epilogue) and this library's
        # GEMM entry on the workload's four projection shapes, stand-alone, each over rotating weight copies; the first
        # launches of a shape run before the timed ones.
        from paper_2602_18447_amd import binding as cb
        T, d, F = wl.T, m.d_model, m.d_ffn
        qkv_n = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
        shapes = [("qkv", T, qkv_n, d, cb.EPI_STORE_F32), ("o_proj", T, d, m.n_q_heads * m.head_dim, cb.EPI_RESID_F32),
                  ("gate_up", T, 2 * F, d, cb.EPI_SWIGLU), ("down", T, d, F, cb.EPI_RESID_F32)]
        ctx = cb.confspec_create(cb.make_model_cfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn,
                                                   m.vocab, m.rope_theta, m.rms_eps, m.dtype))
        res = {}
        for name, M_, N_, K_, epi in shapes:
            A = (torch.randn(M_, K_, device=dev) * 0.5).to(torch.bfloat16)
            Ws = [(torch.randn(N_, K_, device=dev) * 0.02).to(torch.bfloat16) for _ in range(3)]
            out = (torch.empty(M_, N_ // 2, dtype=torch.bfloat16, device=dev) if epi == cb.EPI_SWIGLU
                   else torch.zeros(M_, N_, dtype=torch.float32, device=dev))
            nb = cb.confspec_op_gemm_scratch_bytes(ctx, M_, N_, K_, 1)
            scr = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev) if nb else None

            def timed_us(fn, iters=20):
                for i in range(6):
                    fn(i)
                torch.cuda.synchronize()
                e0.record()
                for i in range(iters):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / iters * 1e3
            rows = {}
            for rep in range(2):                      # twice, alternating, so that neither side always runs first
                rows.setdefault("vendor_us", []).append(timed_us(lambda i: torch.matmul(A, Ws[i % 3].t())))
                rows.setdefault("this_us", []).append(timed_us(lambda i: cb.confspec_op_gemm(ctx, A, Ws[i % 3], out, M_, N_, K_, epi, 1, 1, scr)))
            fl = 2.0 * M_ * N_ * K_
            v, o = min(rows["vendor_us"]), min(rows["this_us"])
            res[name] = dict(M=M_, N=N_, K=K_, vendor_us=round(v, 1), vendor_tflops=round(fl / v / 1e6, 1),
                             this_us=round(o, 1), this_tflops=round(fl / o / 1e6, 1),
                             note="this library's figure includes its fused epilogue (residual add / SwiGLU)")
            del A, Ws, out, scr
        cb.confspec_destroy(ctx)
        extra["vendor_gemm"] = res
    return extra


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0,
                    help="run one workload only: 2, 3, 4 or 5 (default 0: all four, headline on config 4)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP-graph replays")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="confspec_tune setting applied before the run (repeatable), for measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="with --config: also stream 1 GiB through a plain element-wise kernel 6 times, the yardstick for the byte counters")
    ap.add_argument("--cascade", action="store_true",
                    help="with --config: also time the two-tier cascade call (this workload's batch, the 32B-shaped model as "
                         "the large one, gamma 0.9 and 0.6) and report it under \"cascade\"")
    ap.add_argument("--append", type=int, default=0, metavar="N",
                    help="with --config: also time the pass with write-back of the first N suffix tokens of every trace")
    ap.add_argument("--shared-prefix", type=int, default=0, metavar="W",
                    help="with --config: also time the pass with groups of W traces reading the same context pages")
    ap.add_argument("--decode", type=int, default=0, metavar="N",
                    help="with --config: also time N greedy generation steps (one new token per trace)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="with --config: also time the workload's four projection shapes stand-alone, with the vendor BLAS "
                         "library (torch.matmul) and with this library's GEMM entry")
    ap.add_argument("--cpu-baseline-traces", type=int, default=-1,
                    help="traces of the headline workload the CPU oracle is timed on (0 = skip every CPU leg)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (traces are independent; more GPUs would each take a "
              "share of the traces with a replica of the weights, no collectives) - rerun with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2602_18447_amd import binding as cb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    for kv_ in args.tune:
        key, _, val = kv_.partition("=")
        cb.confspec_tune(None, key, int(val))      # defaults of the contexts created below
    configs = [args.config] if args.config else [2, 3, 4, 5]
    headline = args.config if args.config else HEADLINE_CONFIG
    per_config, head_entry, roofline, extra = [], None, None, {}
    for c in configs:
        n_cpu = CPU_SAMPLE.get(c, 2)
        if args.cpu_baseline_traces >= 0 and (c == headline or args.cpu_baseline_traces == 0):
            n_cpu = args.cpu_baseline_traces
        entry, st = _run_config(c, args, dev, n_cpu)
        if c == headline:
            head_entry = entry
            roofline = _roofline(entry, st)
            if args.config:
                extra = _optional_legs(args, st, dev)
        per_config.append(entry)
        print(f"bench.py: {entry['workload']}: {entry['ms_per_step']} ms per pass", file=sys.stderr, flush=True)
        st["ver"].close()
        del st
        torch.cuda.empty_cache()

    h = head_entry
    print(json.dumps({
        "metric": "verified steps/sec (batched verify pass)", "value": h["verified_steps_per_s"],
        "unit": "verified steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": h["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": h["workload"], "B": h["B"], "T": h["T"], "sum_prefix_len": h["sum_prefix_len"],
                   "taus": h["taus"], "accept_counts": h["accept_counts"], "launch": h["launch"],
                   "eager_ms_per_step": h["eager_ms_per_step"], **({"tune": args.tune} if args.tune else {})},
        "roofline": roofline, "cpu_baseline": h["cpu_baseline"],
        "gemm_frac_of_peak": {k: v["frac_of_peak"] for k, v in h["gemm"].items()},
        "per_config": per_config, **extra,
    }))


if __name__ == "__main__":
    main()
