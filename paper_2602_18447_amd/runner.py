"""Device-memory plumbing around the C ABI: owns the context, the packed gate/up
weights, the workspace and the output tensors.  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
from typing import Sequence

import numpy as np
import torch

from . import binding as cb


class Verifier:
    """One model shape on one GPU.

    weights: any object with tensors embed, lm_head, final_norm and per-layer lists attn_norm, wqkv,
    wo, mlp_norm, w_gate_up ([2F, d], gate rows then up rows), w_down - already on the GPU, in the
    model's storage dtype.
    """

    def __init__(self, model_cfg, weights, device: int = 0):
        m = model_cfg
        self.model = m
        self.device = torch.device("cuda", device)
        self.cfg = cb.make_model_cfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn,
                                     m.vocab, m.rope_theta, m.rms_eps, m.dtype)
        self.ctx = cb.confspec_create(self.cfg, device)
        self._weights = weights  # keeps the tensors alive
        w_in, self._keep_in = cb.make_weights(weights.embed, weights.lm_head, weights.final_norm, weights.attn_norm,
                                              weights.wqkv, weights.wo, weights.mlp_norm, weights.w_gate_up,
                                              weights.w_down, packed=0)
        nbytes = cb.confspec_packed_bytes(self.ctx)
        self._packed = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        self._packed_ptrs = (C.c_void_p * max(6 * m.n_layers, 1))()   # pointer arrays of the packed record
        self.w = cb.Weights()
        cb.confspec_pack_weights(self.ctx, w_in, self._packed, nbytes, self._packed_ptrs, self.w)
        torch.cuda.synchronize(self.device)
        self._ws = None

    def close(self):
        if self.ctx is not None:
            cb.confspec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, T: int, B: int) -> torch.Tensor:
        need = cb.confspec_workspace_bytes(self.ctx, T, B, 0)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def bind(self, kv, batch):
        """Builds the KV / batch structs for tensors that already live on the GPU."""
        kvs = cb.make_kv(kv.k_pages, kv.v_pages, batch.block_table, batch.n_blocks, batch.block_size,
                         batch.max_blocks_per_seq)
        bs, keep = cb.make_batch(batch.suffix_ids, batch.cu_suffix, batch.prefix_lens, batch.h_cu_suffix,
                                 batch.h_prefix_lens)
        return kvs, bs, keep

    def alloc_outputs(self, B: int, n_verdict: int, n_tau: int):
        dev = self.device
        return (torch.empty(B, n_verdict, dtype=torch.float32, device=dev),
                torch.empty(B, dtype=torch.float32, device=dev),
                torch.empty(B, dtype=torch.int32, device=dev),
                torch.empty(n_tau, B, dtype=torch.uint8, device=dev))

    def verify(self, kv, batch, verdict_ids: Sequence[int], taus: Sequence[float], outputs=None, stream=None):
        """Enqueues one pass; returns (logits, conf, verdict, accept) device tensors (not synchronised)."""
        kvs, bs, keep = self.bind(kv, batch)
        ws = self.workspace(bs.T, bs.B)
        outs = outputs or self.alloc_outputs(bs.B, len(verdict_ids), len(taus))
        cb.confspec_verify(self.ctx, self.w, kvs, bs, verdict_ids, taus, ws, *outs, stream=stream)
        return outs

    def verify_shared(self, kv, batch, group_start, verdict_ids: Sequence[int], taus: Sequence[float], outputs=None,
                      stream=None):
        """verify() for a batch whose consecutive traces group_start[g] .. group_start[g + 1] - 1 are candidates on one
        shared context (equal prefix lengths, block-table rows naming the same pages)."""
        kvs, bs, keep = self.bind(kv, batch)
        hg = np.ascontiguousarray(group_start, dtype=np.int32)
        dg = torch.from_numpy(hg).to(self.device)
        ws = self.workspace(bs.T, bs.B)
        outs = outputs or self.alloc_outputs(bs.B, len(verdict_ids), len(taus))
        cb.confspec_verify_shared(self.ctx, self.w, kvs, bs, dg, hg, verdict_ids, taus, ws, *outs, stream=stream)
        return outs

    def verify_static(self, kv, batch, verdict_ids: Sequence[int], taus: Sequence[float], outputs, stream=None):
        """verify() on the library's own scratch array: nothing is allocated on the way (the caller brings the
        output tensors).  Batches that need more scratch than the array holds are rejected."""
        kvs, bs, keep = self.bind(kv, batch)
        cb.confspec_verify_static(self.ctx, self.w, kvs, bs, verdict_ids, taus, *outputs, stream=stream)
        return outputs

    def verify_append(self, kv, batch, n_append, verdict_ids: Sequence[int], taus: Sequence[float], outputs=None,
                      stream=None):
        """verify() that also writes the keys / values of the first n_append[b] suffix tokens of every trace into the
        cache pages (kv is modified).  n_append: host integers, one per trace."""
        kvs, bs, keep = self.bind(kv, batch)
        hn = np.ascontiguousarray(n_append, dtype=np.int32)
        dn = torch.from_numpy(hn).to(self.device)
        ws = self.workspace(bs.T, bs.B)
        outs = outputs or self.alloc_outputs(bs.B, len(verdict_ids), len(taus))
        cb.confspec_verify_append(self.ctx, self.w, kvs, bs, dn, hn, verdict_ids, taus, ws, *outs, stream=stream)
        return outs

    def head_scratch(self, B: int) -> torch.Tensor:
        need = cb.confspec_head_scratch_bytes(self.ctx, B)
        if getattr(self, "_head", None) is None or self._head.numel() < need:
            self._head = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._head

    def generate_step(self, kv, batch, n_append=None, verdict_ids=None, outputs=None, stream=None, n_append_dev=None):
        """The pass plus the full-vocabulary head at the last position: returns dict(token, max_logit, lse[, conf_full])
        of device tensors.  n_append: host integers per trace for write-back of the new tokens' keys / values
        (n_append_dev: the same counts already on the device, saves the upload)."""
        kvs, bs, keep = self.bind(kv, batch)
        dev = self.device
        outs = outputs or dict(token=torch.empty(bs.B, dtype=torch.int32, device=dev),
                               max_logit=torch.empty(bs.B, dtype=torch.float32, device=dev),
                               lse=torch.empty(bs.B, dtype=torch.float32, device=dev))
        if verdict_ids is not None and "conf_full" not in outs:
            outs["conf_full"] = torch.empty(bs.B, dtype=torch.float32, device=dev)
        hn = None if n_append is None else np.ascontiguousarray(n_append, dtype=np.int32)
        dn = None if hn is None else (n_append_dev if n_append_dev is not None else torch.from_numpy(hn).to(dev))
        ho = cb.HeadOut(outs["token"].data_ptr(), outs["max_logit"].data_ptr(), outs["lse"].data_ptr(),
                        outs["conf_full"].data_ptr() if verdict_ids is not None else None)
        cb.confspec_generate_step(self.ctx, self.w, kvs, bs, dn, hn, verdict_ids, self.workspace(bs.T, bs.B),
                                  self.head_scratch(bs.B), ho, stream=stream)
        return outs

    def generate_greedy(self, kv, block_table, n_blocks: int, max_blocks_per_seq: int, first_ids, prefix_lens, n_steps: int):
        """n_steps greedy tokens per trace on a growing cache, one token per trace and step; nothing here waits for the
        GPU.  first_ids: device int32 [B], the token at position L_b (not cached yet); prefix_lens: host integers.
        The block table must cover L_b + n_steps rows.  Returns (tokens [n_steps, B], max_logit, lse) device tensors."""
        from types import SimpleNamespace
        dev = self.device
        B = len(prefix_lens)
        L0 = np.ascontiguousarray(prefix_lens, dtype=np.int32)
        toks = torch.empty(n_steps, B, dtype=torch.int32, device=dev)
        zmax = torch.empty(n_steps, B, dtype=torch.float32, device=dev)
        lse = torch.empty(n_steps, B, dtype=torch.float32, device=dev)
        cu = np.arange(B + 1, dtype=np.int32)
        cu_dev = torch.from_numpy(cu).to(dev)
        ones = np.ones(B, dtype=np.int32)
        ones_dev = torch.from_numpy(ones).to(dev)
        # every step's context lengths, uploaded once: a copy from pageable host memory inside the loop would make
        # each step wait for the one before
        lens_host = L0[None, :] + np.arange(n_steps, dtype=np.int32)[:, None]
        lens_dev = torch.from_numpy(np.ascontiguousarray(lens_host)).to(dev)
        cur = first_ids
        for i in range(n_steps):
            batch = SimpleNamespace(suffix_ids=cur, cu_suffix=cu_dev, prefix_lens=lens_dev[i],
                                    block_table=block_table, n_blocks=n_blocks, max_blocks_per_seq=max_blocks_per_seq,
                                    block_size=kv.block_size, h_cu_suffix=cu, h_prefix_lens=lens_host[i])
            self.generate_step(kv, batch, n_append=ones, n_append_dev=ones_dev,
                               outputs=dict(token=toks[i], max_logit=zmax[i], lse=lse[i]))
            cur = toks[i]
        return toks, zmax, lse


class Cascade:
    """The two-tier cascade over the drafted steps of a batch of requests: a small and a large Verifier that read
    the same token ids, each with its own cache of the same contexts.  Only buffers are owned here."""

    NAMES = ("conf_draft", "verdict_draft", "conf_target", "verdict_target", "decision", "escalated", "target_ran",
             "accepted_steps", "selected", "conf_used")

    def __init__(self, draft: Verifier, target: Verifier):
        self.draft, self.target = draft, target
        self._scratch = None

    def alloc_outputs(self, B: int, R: int):
        dev = self.draft.device
        f32, i32, u8 = torch.float32, torch.int32, torch.uint8
        dts = (f32, i32, f32, i32, i32, u8, u8, i32, u8, f32)
        return {n: torch.empty(R if n == "accepted_steps" else B, dtype=dt, device=dev) for n, dt in zip(self.NAMES, dts)}

    def run(self, draft_kv, target_kv, batch, h_req_start, verdict_ids: Sequence[int], gamma: float, outputs=None,
            stream=None, parent=None):
        """One cascade; synchronises the stream once inside.  parent: host integers [B] for candidate trees, None for
        chains.  Returns (outputs dict of device tensors, traces the large model's pass held)."""
        kd, bs, keep = self.draft.bind(draft_kv, batch)
        kt, _, keep_t = self.target.bind(target_kv, batch)
        hr = np.ascontiguousarray(h_req_start, dtype=np.int32)
        req_dev = torch.from_numpy(hr).to(self.draft.device)
        hp = None if parent is None else np.ascontiguousarray(parent, dtype=np.int32)
        par_dev = None if hp is None else torch.from_numpy(hp).to(self.draft.device)
        reqs, keep_r = cb.make_requests(req_dev, hr, par_dev, hp)
        need = cb.confspec_cascade_scratch_bytes(bs.B, bs.T, kt.max_blocks_per_seq)
        if self._scratch is None or self._scratch.numel() < need:
            self._scratch = torch.empty(need, dtype=torch.uint8, device=self.draft.device)
        outs = outputs or self.alloc_outputs(bs.B, len(hr) - 1)
        co = cb.CascadeOut(*[outs[n].data_ptr() for n in self.NAMES])
        n_target = cb.confspec_cascade(self.draft.ctx, self.draft.w, kd, self.draft.workspace(bs.T, bs.B),
                                       self.target.ctx, self.target.w, kt, self.target.workspace(bs.T, bs.B), bs, reqs,
                                       verdict_ids, gamma, self._scratch, co, stream=stream)
        return outs, n_target
