"""Shared driver for end-to-end GPU parity cases: build seeded inputs on the GPU, run the HIP path
through the C ABI, run the CPU oracle on the very same (already rounded) tensors, compare."""
import time

import numpy as np
import torch

import confspec_workloads as W
from oracle import confspec_oracle as O
from paper_2602_18447_amd.runner import Verifier

DEV = "cuda:0"

# Bounds of the comparison (absolute): verdict logits, confidence, and the band around tau inside
# which gate decisions are not compared.  bf16 figures are the stated targets; the fp32 ones follow
# from fp32 accumulation over at most a few thousand terms of O(1) products.
TOL = {"bf16": dict(logit=2e-2, conf=1e-2, band=1e-2), "fp32": dict(logit=1e-4, conf=1e-5, band=1e-5)}


def build_inputs(wl, device=DEV):
    weights = W.make_weights(wl.model, wl.seed, device)
    batch = W.make_batch(wl, device)
    if wl.kv_source == "prefix_pass":
        kd, vd = O.prefix_pass(wl.model, W.OracleModelView(weights), W.make_prefix_ids(wl))
        kv = W.pages_from_dense(wl, batch, kd, vd, device)
    else:
        kv = W.make_seeded_kv(wl, batch, device)
    return weights, batch, kv


def run_gpu(wl, weights, batch, kv, taus=None, verifier=None):
    taus = list(taus if taus is not None else wl.taus)
    vids = W.draw_verdict_ids(wl)
    own = verifier is None
    ver = verifier or Verifier(wl.model, weights)
    logits, conf, verdict, accept = ver.verify(kv, batch, vids, taus)
    torch.cuda.synchronize()
    res = dict(logits=logits.cpu().numpy().astype(np.float64), conf=conf.cpu().numpy().astype(np.float64),
               verdict=verdict.cpu().numpy(), accept=accept.cpu().numpy(), taus=taus, vids=vids)
    if own:
        ver.close()
    return res


def run_oracle(wl, weights, batch, kv, taus, vids, traces=None):
    return O.verify(wl.model, W.OracleModelView(weights), W.OracleKVView(kv, batch), wl.block_size,
                    batch.suffix_ids.cpu().numpy(), batch.h_cu_suffix, batch.h_prefix_lens, vids, taus,
                    trace_subset=traces)


def compare(wl, gpu, ora, label=""):
    """Element-by-element comparison on the traces the oracle computed.  Returns a summary dict."""
    tol = TOL[wl.model.dtype]
    tr = ora["traces"]
    dl = np.abs(gpu["logits"][tr] - ora["logits"])
    dc = np.abs(gpu["conf"][tr] - ora["conf"])
    mism = 0
    compared = 0
    kept = 0                       # compared (trace, tau) pairs whose decision is kept; the rest escalate
    for i, tau in enumerate(gpu["taus"]):
        clear = np.abs(ora["conf"] - tau) > tol["band"]
        compared += int(clear.sum())
        kept += int(ora["accept"][i][clear].sum())
        mism += int((gpu["accept"][i][tr][clear] != ora["accept"][i][clear]).sum())
    srt = np.sort(ora["logits"], axis=1)
    decided = (srt[:, -1] - srt[:, -2]) > 2 * tol["logit"]
    vmis = int((gpu["verdict"][tr][decided] != ora["verdict"][decided]).sum())
    summary = dict(label=label, traces=len(tr), max_dlogit=float(dl.max()), max_dconf=float(dc.max()),
                   gate_compared=compared, gate_kept=kept, gate_escalated=compared - kept, gate_mismatch=mism,
                   verdict_mismatch=vmis,
                   accept_counts=[int(a.sum()) for a in gpu["accept"]])
    print("parity", summary, flush=True)
    assert dl.max() <= tol["logit"], summary
    assert dc.max() <= tol["conf"], summary
    assert mism == 0 and vmis == 0, summary
    # properties that hold for every trace at any size
    assert np.all(gpu["conf"] >= 1.0 / gpu["logits"].shape[1] - 1e-6) and np.all(gpu["conf"] <= 1.0 + 1e-6)
    order = np.argsort(gpu["taus"])
    acc = gpu["accept"][order]
    assert np.all(acc[1:] <= acc[:-1]), "accept set must shrink as tau rises"
    return summary


# Thresholds for the full-size cases: the workload's own plus a sweep through the range where random-init
# confidences fall (0.5 .. 0.7), so that kept and escalated decisions both occur among the compared traces.
SWEEP_TAUS = (0.52, 0.55, 0.6, 0.7)


def sweep_taus(wl):
    return sorted(set(float(t) for t in wl.taus) | set(SWEEP_TAUS))


def parity_case(wl, traces=None, taus=None, label=None):
    t0 = time.time()
    weights, batch, kv = build_inputs(wl)
    t1 = time.time()
    gpu = run_gpu(wl, weights, batch, kv, taus)
    t2 = time.time()
    ora = run_oracle(wl, weights, batch, kv, gpu["taus"], gpu["vids"], traces)
    t3 = time.time()
    print(f"{label or wl.name}: inputs {t1 - t0:.1f}s gpu {t2 - t1:.1f}s oracle {t3 - t2:.1f}s", flush=True)
    return compare(wl, gpu, ora, label or wl.name), gpu, ora
