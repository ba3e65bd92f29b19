"""Seeded synthetic workloads: decoder weights, paged prefix KV, ragged batches.

Everything here is input generation: random draws keyed by (seed, tensor name),
round-to-nearest-even casts to the storage dtype, block-table construction and
byte movement between dense and paged layouts.  No normalisation, rotation,
attention, softmax or gating is computed in this module.

The model shapes stand in for the two model sizes the paper pairs (a ~1.5B
draft and a 32B target, Section 5.1 "Models"); token ids are uniform random
because neither the verification prompt nor the verdict token ids are printed
in the paper (Section 4.2 only says "e.g. Yes / No").
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch


# --------------------------------------------------------------------------- #
# configuration records
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    dtype: str = "bf16"  # storage dtype of weights and KV pages: "bf16" | "fp32"

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelCfg
    seed: int
    prefix_lens: Tuple[int, ...]
    suffix_lens: Tuple[int, ...]
    block_size: int = 16
    n_verdict: int = 2
    taus: Tuple[float, ...] = (0.9,)
    # "seeded": KV pages are filled with seeded values directly.
    # "prefix_pass": the caller fills the cache from a real prefix pass over
    #                `make_prefix_ids` (done with the CPU oracle in the tests).
    kv_source: str = "seeded"

    @property
    def B(self) -> int:
        return len(self.prefix_lens)

    @property
    def T(self) -> int:
        return int(sum(self.suffix_lens))


def torch_dtype(name: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp32": torch.float32}[name]


def _key(seed: int, tag: str) -> int:
    """63-bit stream key for (seed, tensor name); stable across hosts."""
    h = hashlib.blake2b(f"{seed}/{tag}".encode(), digest_size=8).digest()
    return int.from_bytes(h, "little") & ((1 << 63) - 1)


def _np_rng(seed: int, tag: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=_key(seed, tag)))


DRAFT_SHAPE = ModelCfg(n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128,
                       d_ffn=8960, vocab=151936, dtype="bf16")
TARGET_SHAPE = ModelCfg(n_layers=64, d_model=5120, n_q_heads=40, n_kv_heads=8, head_dim=128,
                        d_ffn=27648, vocab=152064, dtype="bf16")
TINY_FP32 = ModelCfg(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                     d_ffn=1024, vocab=4096, dtype="fp32")


def config(i: int) -> Workload:
    """The five benchmark configurations (1-based)."""
    if i == 1:
        return Workload("cfg1_tiny_fp32", TINY_FP32, 1001, (128,) * 4, (32,) * 4,
                        taus=(0.9,), kv_source="prefix_pass")
    if i == 2:
        return Workload("cfg2_draft_b32_L2048_S96", DRAFT_SHAPE, 1002, (2048,) * 32, (96,) * 32)
    if i == 3:
        return Workload("cfg3_draft_b64_L8192_S128", DRAFT_SHAPE, 1003, (8192,) * 64, (128,) * 64,
                        taus=(0.8, 0.9, 0.95))
    if i == 4:
        rng = _np_rng(1004, "lengths")
        L = rng.integers(512, 16384 + 1, size=128)
        S = rng.integers(32, 256 + 1, size=128)
        return Workload("cfg4_draft_ragged_b128", DRAFT_SHAPE, 1004,
                        tuple(int(v) for v in L), tuple(int(v) for v in S))
    if i == 5:
        return Workload("cfg5_target_b16_L4096_S96", TARGET_SHAPE, 1005, (4096,) * 16, (96,) * 16)
    raise ValueError(f"no config {i}")


def tiny_workload(name: str, seed: int, *, dtype: str = "fp32", n_layers: int = 2, d_model: int = 64,
                  n_q_heads: int = 4, n_kv_heads: int = 2, head_dim: int = 16, d_ffn: int = 128,
                  vocab: int = 97, prefix_lens: Sequence[int] = (5, 0, 19),
                  suffix_lens: Sequence[int] = (3, 1, 7), block_size: int = 4,
                  taus: Sequence[float] = (0.9,), n_verdict: int = 2,
                  kv_source: str = "seeded", rope_theta: float = 1.0e6) -> Workload:
    """Small free-form workload for CPU tests and reduced-size GPU parity cases."""
    m = ModelCfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                 rope_theta=rope_theta, dtype=dtype)
    return Workload(name, m, seed, tuple(prefix_lens), tuple(suffix_lens), block_size=block_size,
                    n_verdict=n_verdict, taus=tuple(taus), kv_source=kv_source)


# --------------------------------------------------------------------------- #
# tensors
# --------------------------------------------------------------------------- #
def _normal(seed: int, tag: str, shape, std: float, mean: float, dtype: torch.dtype,
            device) -> torch.Tensor:
    """N(mean, std) drawn in fp32 on `device`, then rounded (RNE) to `dtype`."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(_key(seed, tag))
    t = torch.randn(shape, generator=g, dtype=torch.float32, device=dev)
    t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(dtype)


@dataclass
class Weights:
    """Row-major [out, in] matrices in the model's storage dtype.

    wqkv[l]      : [(Hq + 2 Hkv) * hd, d]  rows = q heads, then k heads, then v heads
    wo[l]        : [d, Hq * hd]
    w_gate_up[l] : [2 F, d]                rows 0..F-1 = gate, rows F..2F-1 = up
    w_down[l]    : [d, F]
    """
    cfg: ModelCfg
    embed: torch.Tensor
    lm_head: torch.Tensor
    final_norm: torch.Tensor
    attn_norm: List[torch.Tensor] = field(default_factory=list)
    wqkv: List[torch.Tensor] = field(default_factory=list)
    wo: List[torch.Tensor] = field(default_factory=list)
    mlp_norm: List[torch.Tensor] = field(default_factory=list)
    w_gate_up: List[torch.Tensor] = field(default_factory=list)
    w_down: List[torch.Tensor] = field(default_factory=list)


def make_weights(cfg: ModelCfg, seed: int, device="cpu", std: float = 0.02) -> Weights:
    """Matrices and embeddings ~ N(0, std); norm gains ~ 1 + N(0, std)."""
    dt = torch_dtype(cfg.dtype)
    d, F = cfg.d_model, cfg.d_ffn
    w = Weights(
        cfg,
        embed=_normal(seed, "embed", (cfg.vocab, d), std, 0.0, dt, device),
        lm_head=_normal(seed, "lm_head", (cfg.vocab, d), std, 0.0, dt, device),
        final_norm=_normal(seed, "final_norm", (d,), std, 1.0, dt, device),
    )
    for l in range(cfg.n_layers):
        w.attn_norm.append(_normal(seed, f"L{l}.attn_norm", (d,), std, 1.0, dt, device))
        w.wqkv.append(_normal(seed, f"L{l}.wqkv", (cfg.qkv_rows, d), std, 0.0, dt, device))
        w.wo.append(_normal(seed, f"L{l}.wo", (d, cfg.n_q_heads * cfg.head_dim), std, 0.0, dt, device))
        w.mlp_norm.append(_normal(seed, f"L{l}.mlp_norm", (d,), std, 1.0, dt, device))
        w.w_gate_up.append(_normal(seed, f"L{l}.w_gate_up", (2 * F, d), std, 0.0, dt, device))
        w.w_down.append(_normal(seed, f"L{l}.w_down", (d, F), std, 0.0, dt, device))
    return w


@dataclass
class Batch:
    suffix_ids: torch.Tensor      # int32 [T], packed over traces
    cu_suffix: torch.Tensor       # int32 [B+1], exclusive prefix sums of S_b
    prefix_lens: torch.Tensor     # int32 [B]
    block_table: torch.Tensor     # int32 [B, max_blocks_per_seq]
    n_blocks: int                 # physical blocks in the cache
    max_blocks_per_seq: int
    block_size: int
    h_cu_suffix: np.ndarray       # host copies (int32)
    h_prefix_lens: np.ndarray


def make_batch(wl: Workload, device="cpu", spare_blocks: int = 3, extra_rows=0) -> Batch:
    """Uniform random suffix ids; physical blocks handed out by a seeded permutation.
    extra_rows (int or one per trace): rows past the prefix that the block table also covers, for callers
    that append to the cache."""
    V = wl.model.vocab
    rng = _np_rng(wl.seed, "batch")
    S = np.asarray(wl.suffix_lens, dtype=np.int64)
    L = np.asarray(wl.prefix_lens, dtype=np.int64)
    cu = np.zeros(wl.B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(S)
    ids = rng.integers(0, V, size=int(cu[-1]), dtype=np.int64).astype(np.int32)
    bs = wl.block_size
    need = (L + np.broadcast_to(np.asarray(extra_rows, dtype=np.int64), L.shape) + bs - 1) // bs
    n_blocks = int(need.sum()) + spare_blocks
    max_blocks = max(1, int(need.max()) if len(need) else 1)
    perm = rng.permutation(n_blocks).astype(np.int32)
    table = np.zeros((wl.B, max_blocks), dtype=np.int32)
    at = 0
    for b in range(wl.B):
        table[b, : need[b]] = perm[at: at + need[b]]
        at += int(need[b])
    dev = torch.device(device)
    return Batch(
        suffix_ids=torch.from_numpy(ids).to(dev),
        cu_suffix=torch.from_numpy(cu).to(dev),
        prefix_lens=torch.from_numpy(L.astype(np.int32)).to(dev),
        block_table=torch.from_numpy(table).to(dev),
        n_blocks=n_blocks,
        max_blocks_per_seq=max_blocks,
        block_size=bs,
        h_cu_suffix=cu,
        h_prefix_lens=L.astype(np.int32),
    )


def draw_verdict_ids(wl: Workload) -> np.ndarray:
    """n_verdict distinct token ids; index 0 plays "Yes" (accept the step), 1 plays "No"."""
    rng = _np_rng(wl.seed, "verdict")
    return rng.choice(wl.model.vocab, size=wl.n_verdict, replace=False).astype(np.int32)


def make_prefix_ids(wl: Workload) -> List[np.ndarray]:
    """Uniform random context token ids per trace (for caches built by a real prefix pass)."""
    rng = _np_rng(wl.seed, "prefix_ids")
    return [rng.integers(0, wl.model.vocab, size=int(L), dtype=np.int64).astype(np.int32)
            for L in wl.prefix_lens]


@dataclass
class KVCache:
    """k_pages, v_pages: [n_layers, n_blocks, H_kv, block_size, head_dim], storage dtype."""
    k_pages: torch.Tensor
    v_pages: torch.Tensor
    block_size: int


def make_seeded_kv(wl: Workload, batch: Batch, device="cpu", scale: float = 0.5) -> KVCache:
    """Pages filled with N(0, scale) values: a stand-in for a real cached context."""
    m = wl.model
    dt = torch_dtype(m.dtype)
    shape = (m.n_layers, batch.n_blocks, m.n_kv_heads, wl.block_size, m.head_dim)
    k = torch.empty(shape, dtype=dt, device=device)
    v = torch.empty(shape, dtype=dt, device=device)
    for l in range(m.n_layers):
        k[l].copy_(_normal(wl.seed, f"L{l}.k_pages", shape[1:], scale, 0.0, dt, device))
        v[l].copy_(_normal(wl.seed, f"L{l}.v_pages", shape[1:], scale, 0.0, dt, device))
    return KVCache(k, v, wl.block_size)


def pages_from_dense(wl: Workload, batch: Batch, k_dense, v_dense, device="cpu") -> KVCache:
    """Scatter dense per-trace caches into pages through the block table.

    k_dense[l][b], v_dense[l][b]: array-like [L_b, H_kv, head_dim] (any float dtype);
    values are rounded to the storage dtype on the way in.  Unused slots stay zero.
    """
    m = wl.model
    dt = torch_dtype(m.dtype)
    bs = wl.block_size
    shape = (m.n_layers, batch.n_blocks, m.n_kv_heads, bs, m.head_dim)
    k = torch.zeros(shape, dtype=dt)
    v = torch.zeros(shape, dtype=dt)
    table = batch.block_table.cpu().numpy()
    for l in range(m.n_layers):
        for b, L in enumerate(wl.prefix_lens):
            kd = torch.as_tensor(np.asarray(k_dense[l][b])).to(dt)
            vd = torch.as_tensor(np.asarray(v_dense[l][b])).to(dt)
            for j in range(L):
                blk, slot = int(table[b, j // bs]), j % bs
                k[l, blk, :, slot, :] = kd[j]
                v[l, blk, :, slot, :] = vd[j]
    return KVCache(k.to(device), v.to(device), bs)


# --------------------------------------------------------------------------- #
# fp64 views handed to the CPU oracle (dtype widening only)
# --------------------------------------------------------------------------- #
def _f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


class OracleModelView:
    """Widens the stored (already rounded) weights to float64 numpy, lazily."""

    def __init__(self, w: Weights):
        self._w = w
        self.cfg = w.cfg

    @property
    def final_norm(self) -> np.ndarray:
        return _f64(self._w.final_norm)

    def embed_rows(self, ids) -> np.ndarray:
        idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=self._w.embed.device)
        return _f64(self._w.embed[idx])

    def lm_head_rows(self, ids) -> np.ndarray:
        idx = torch.as_tensor(np.asarray(ids, dtype=np.int64), device=self._w.lm_head.device)
        return _f64(self._w.lm_head[idx])

    def lm_head_full(self) -> np.ndarray:
        return _f64(self._w.lm_head)

    def layer(self, l: int) -> dict:
        c, w = self.cfg, self._w
        nq, nkv = c.n_q_heads * c.head_dim, c.n_kv_heads * c.head_dim
        qkv = _f64(w.wqkv[l])
        gu = _f64(w.w_gate_up[l])
        return dict(
            attn_norm=_f64(w.attn_norm[l]),
            wq=qkv[:nq], wk=qkv[nq:nq + nkv], wv=qkv[nq + nkv:],
            wo=_f64(w.wo[l]),
            mlp_norm=_f64(w.mlp_norm[l]),
            wg=gu[: c.d_ffn], wu=gu[c.d_ffn:],
            wd=_f64(w.w_down[l]),
        )


class OracleKVView:
    """Widens selected physical blocks of one layer to float64 numpy."""

    def __init__(self, kv: KVCache, batch: Batch):
        self._kv = kv
        self.block_size = kv.block_size
        self.block_table = batch.block_table.detach().cpu().numpy()

    def _blocks(self, pages: torch.Tensor, l: int, block_ids) -> np.ndarray:
        idx = torch.as_tensor(np.asarray(block_ids, dtype=np.int64), device=pages.device)
        return _f64(pages[l][idx])  # [n, H_kv, block_size, head_dim]

    def k_blocks(self, l: int, block_ids) -> np.ndarray:
        return self._blocks(self._kv.k_pages, l, block_ids)

    def v_blocks(self, l: int, block_ids) -> np.ndarray:
        return self._blocks(self._kv.v_pages, l, block_ids)
