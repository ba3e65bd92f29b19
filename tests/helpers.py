"""Small helpers shared by the CPU tests (no method arithmetic here)."""
import types

import numpy as np


class DictModel:
    """float64 model held as plain numpy arrays so tests can edit single matrices."""

    def __init__(self, cfg, seed=0, std=0.3):
        rng = np.random.default_rng(seed)
        c = cfg
        nq, nkv = c.n_q_heads * c.head_dim, c.n_kv_heads * c.head_dim
        self.cfg = c
        self.embed = rng.normal(0, 1.0, (c.vocab, c.d_model))
        self.lm_head = rng.normal(0, std, (c.vocab, c.d_model))
        self.final_norm = 1 + rng.normal(0, 0.2, c.d_model)
        self.layers = []
        for _ in range(c.n_layers):
            self.layers.append(dict(
                attn_norm=1 + rng.normal(0, 0.2, c.d_model),
                wq=rng.normal(0, std, (nq, c.d_model)),
                wk=rng.normal(0, std, (nkv, c.d_model)),
                wv=rng.normal(0, std, (nkv, c.d_model)),
                wo=rng.normal(0, std, (c.d_model, nq)),
                mlp_norm=1 + rng.normal(0, 0.2, c.d_model),
                wg=rng.normal(0, std, (c.d_ffn, c.d_model)),
                wu=rng.normal(0, std, (c.d_ffn, c.d_model)),
                wd=rng.normal(0, std, (c.d_model, c.d_ffn)),
            ))

    def embed_rows(self, ids):
        return self.embed[np.asarray(ids, dtype=np.int64)]

    def lm_head_rows(self, ids):
        return self.lm_head[np.asarray(ids, dtype=np.int64)]

    def lm_head_full(self):
        return self.lm_head

    def layer(self, l):
        return self.layers[l]


def small_cfg(**kw):
    base = dict(n_layers=2, d_model=8, n_q_heads=2, n_kv_heads=1, head_dim=4, d_ffn=12, vocab=23,
                rope_theta=1.0e6, rms_eps=1.0e-6)
    base.update(kw)
    return types.SimpleNamespace(**base)


class DenseKV:
    """Paged view over dense per-trace caches with an arbitrary block assignment."""

    def __init__(self, k_dense, v_dense, prefix_lens, block_size, n_kv_heads, head_dim, perm_seed=0):
        # k_dense[l][b]: [L_b, Hkv, hd]
        self.block_size = bs = block_size
        n_layers = len(k_dense)
        need = [(L + bs - 1) // bs for L in prefix_lens]
        n_blocks = sum(need) + 2
        rng = np.random.default_rng(perm_seed)
        perm = rng.permutation(n_blocks)
        self.block_table = np.zeros((len(prefix_lens), max(1, max(need, default=1))), dtype=np.int32)
        at = 0
        for b, n in enumerate(need):
            self.block_table[b, :n] = perm[at:at + n]
            at += n
        self.k = np.full((n_layers, n_blocks, n_kv_heads, bs, head_dim), np.nan)
        self.v = np.full((n_layers, n_blocks, n_kv_heads, bs, head_dim), np.nan)
        for l in range(n_layers):
            for b, L in enumerate(prefix_lens):
                for j in range(L):
                    blk = self.block_table[b, j // bs]
                    self.k[l, blk, :, j % bs, :] = k_dense[l][b][j]
                    self.v[l, blk, :, j % bs, :] = v_dense[l][b][j]
        # unused slots hold NaN on purpose: reading one poisons the result
        self.k_used = self.k
        self.v_used = self.v

    def k_blocks(self, l, ids):
        return np.nan_to_num(self.k[l][np.asarray(ids, dtype=np.int64)], nan=1e30)

    def v_blocks(self, l, ids):
        return np.nan_to_num(self.v[l][np.asarray(ids, dtype=np.int64)], nan=1e30)
