"""Per-step GPU parity: each kernel of the pass against the matching oracle sub-step, through the C ABI.

Inputs are rounded to the storage dtype first and the oracle reads exactly those values (widened to
fp64), so differences come from the kernels' own arithmetic only.  Tolerances: fp32 steps accumulate
in fp32 (1e-5 relative to the result scale); bf16 GEMMs accumulate in fp32, so an fp32 output carries
about sqrt(K) * 2^-24 of the product scale and a bf16 output one rounding (2^-9 relative); bf16
attention additionally rounds the probabilities to bf16 before P.V.
"""
import numpy as np
import pytest
import torch

import confspec_workloads as W
from oracle import confspec_oracle as O
from paper_2602_18447_amd import binding as cb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def _ctx(dtype, **kw):
    base = dict(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=256, vocab=512,
                rope_theta=1e6, rms_eps=1e-6, dtype=dtype)
    base.update(kw)
    return cb.confspec_create(cb.make_model_cfg(**base)), base


def _rand(shape, dtype, seed, scale=1.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn(shape, generator=g, device=DEV, dtype=torch.float32) * scale).to(dtype)


def _pack_rows(F):
    p = np.arange(2 * F)
    blk, w = p // 64, p % 64
    f = blk * 32 + (w % 32)
    return np.where(w < 32, f, F + f)


# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("tile", [1, 4, 7])
@pytest.mark.parametrize("M,N,K", [(300, 512, 192), (1, 256, 64), (257, 768, 1024), (512, 256, 320), (400, 384, 128),
                                   (300, 512, 128), (259, 256, 256), (700, 512, 384)])   # 2, 4 and 6 k-tiles: the ring's first rounds
def test_gemm_bf16_store_and_residual(tile, M, N, K):
    print(f"gemm bf16 tile={tile} M={M} N={N} K={K}", flush=True)
    ctx, _ = _ctx("bf16")
    cb.confspec_tune(ctx, "gemm_tile", tile)
    A = _rand((M, K), torch.bfloat16, 1)
    Wt = _rand((N, K), torch.bfloat16, 2, 0.05)
    ref = f64(A) @ f64(Wt).T
    scale = np.abs(ref).max()
    out = torch.full((M + 3, N), 7.0, dtype=torch.float32, device=DEV)       # 3 guard rows
    cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, cb.EPI_STORE_F32)
    torch.cuda.synchronize()
    assert np.abs(f64(out[:M]) - ref).max() <= 2e-5 * scale
    assert torch.all(out[M:] == 7.0)
    x0 = _rand((M, N), torch.float32, 3)
    x = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32)
    torch.cuda.synchronize()
    assert np.abs(f64(x) - (f64(x0) + ref)).max() <= 2e-5 * max(scale, 4.0)
    cb.confspec_destroy(ctx)


def test_gemm_bf16_seeded_random_shapes():
    """48 seeded shapes (rows 1..900, 128..1280 columns, 1..20 k-tiles), every tile choice, store / residual epilogue,
    bf16 and fp16 operands, with and without split-K scratch: every element against the fp64 product."""
    rng = np.random.default_rng(20260218)
    ctx, _ = _ctx("bf16")
    for case in range(48):
        M = int(rng.integers(1, 901))
        N = 128 * int(rng.integers(1, 11))
        K = 64 * int(rng.integers(1, 21))
        tile = int(rng.choice([0, 1, 4, 7]))
        epi = int(rng.choice([cb.EPI_STORE_F32, cb.EPI_RESID_F32]))
        f16 = bool(rng.integers(0, 2))
        with_scratch = bool(rng.integers(0, 2))
        print(f"case {case}: M={M} N={N} K={K} tile={tile} epi={epi} f16={f16} scratch={with_scratch}", flush=True)
        cb.confspec_tune(ctx, "gemm_tile", tile)
        dt = torch.float16 if f16 else torch.bfloat16
        A = _rand((M, K), dt, 1000 + case)
        Wt = _rand((N, K), dt, 2000 + case, 0.05)
        ref = f64(A) @ f64(Wt).T
        x0 = _rand((M + 2, N), torch.float32, 3000 + case)           # two guard rows
        out = x0.clone()
        scr = None
        if with_scratch and tile == 0:
            nb = cb.confspec_op_gemm_scratch_bytes(ctx, M, N, K, 3 if f16 else 1)
            scr = torch.empty(max(nb, 16), dtype=torch.uint8, device=DEV) if nb else None
        cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, epi, 3 if f16 else 1, 1, scr)
        torch.cuda.synchronize()
        want = ref + (f64(x0[:M]) if epi == cb.EPI_RESID_F32 else 0.0)
        assert np.abs(f64(out[:M]) - want).max() <= 2e-5 * max(np.abs(ref).max(), 4.0), case
        assert torch.equal(out[M:], x0[M:]), case
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("tile", [1, 4])
def test_gemm_bf16_swiglu_epilogue(tile):
    print(f"gemm bf16 swiglu tile={tile}", flush=True)
    ctx, _ = _ctx("bf16")
    cb.confspec_tune(ctx, "gemm_tile", tile)
    M, F, K = 200, 384, 256
    A = _rand((M, K), torch.bfloat16, 4)
    Wgu = _rand((2 * F, K), torch.bfloat16, 5, 0.1)           # gate rows, then up rows
    packed = Wgu[torch.as_tensor(_pack_rows(F), device=DEV)].contiguous()
    out = torch.zeros((M, F), dtype=torch.bfloat16, device=DEV)
    cb.confspec_op_gemm(ctx, A, packed, out, M, 2 * F, K, cb.EPI_SWIGLU)
    torch.cuda.synchronize()
    g = f64(A) @ f64(Wgu[:F]).T
    u = f64(A) @ f64(Wgu[F:]).T
    ref = O.silu(g) * u
    err = np.abs(f64(out) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-4 * np.abs(ref).max())
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("tile", [0, 4])      # 4: the 256 x 256 tile's pipeline with the hi / lo k-tiles alternating
def test_two_term_activations_through_gemm_rmsnorm_and_swiglu(tile):
    """hi | lo operands: the GEMM must return (hi + lo) . W^T, i.e. the product with the activation
    kept to 16 mantissa bits, and the producers must emit hi = bf16(v), lo = bf16(v - hi)."""
    print(f"two-term activations, tile {tile}", flush=True)
    d = 512
    ctx, base = _ctx("bf16", d_model=d)
    cb.confspec_tune(ctx, "gemm_tile", tile)
    M, N, K = 150, 512, d
    x = _rand((M, d), torch.float32, 40, 2.0)
    g = (1 + 0.1 * _rand((d,), torch.float32, 41)).to(torch.bfloat16)
    h2 = torch.zeros((M, 2 * d), dtype=torch.bfloat16, device=DEV)
    cb.confspec_op_rmsnorm(ctx, x, g, h2, M, out_terms=2)
    torch.cuda.synchronize()
    ref_h = O.rmsnorm(f64(x), f64(g), base["rms_eps"])
    hi, lo = f64(h2[:, :d]), f64(h2[:, d:])
    assert np.all(np.abs(hi - ref_h) <= 2.0 ** -8 * np.abs(ref_h) + 1e-7)
    assert np.all(np.abs(hi + lo - ref_h) <= 2.0 ** -15 * np.abs(ref_h) + 1e-6)   # fp32 evaluation of the norm
    Wt = _rand((N, K), torch.bfloat16, 42, 0.05)
    out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    cb.confspec_op_gemm(ctx, h2, Wt, out, M, N, K, cb.EPI_STORE_F32, a_terms=2)
    torch.cuda.synchronize()
    ref = (hi + lo) @ f64(Wt).T
    assert np.abs(f64(out) - ref).max() <= 2e-5 * np.abs(ref).max()
    one = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    cb.confspec_op_gemm(ctx, h2[:, :d].contiguous(), Wt, one, M, N, K, cb.EPI_STORE_F32)
    torch.cuda.synchronize()
    exact = ref_h @ f64(Wt).T
    assert np.abs(f64(out) - exact).max() < 0.1 * np.abs(f64(one) - exact).max()
    # SwiGLU epilogue producing hi | lo
    F = 256
    Wgu = _rand((2 * F, K), torch.bfloat16, 43, 0.1)
    packed = Wgu[torch.as_tensor(_pack_rows(F), device=DEV)].contiguous()
    act2 = torch.zeros((M, 2 * F), dtype=torch.bfloat16, device=DEV)
    cb.confspec_op_gemm(ctx, h2, packed, act2, M, 2 * F, K, cb.EPI_SWIGLU, a_terms=2, out_terms=2)
    torch.cuda.synchronize()
    gate, up = (hi + lo) @ f64(Wgu[:F]).T, (hi + lo) @ f64(Wgu[F:]).T
    ref_act = O.silu(gate) * up
    got = f64(act2[:, :F]) + f64(act2[:, F:])
    assert np.abs(got - ref_act).max() <= 3e-5 * np.abs(ref_act).max()
    cb.confspec_destroy(ctx)


def test_gemm_fp32_all_epilogues():
    print("gemm fp32", flush=True)
    ctx, _ = _ctx("fp32", head_dim=64, n_kv_heads=4)
    M, N, K = 77, 192, 80
    A = _rand((M, K), torch.float32, 6)
    Wt = _rand((N, K), torch.float32, 7, 0.1)
    ref = f64(A) @ f64(Wt).T
    out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, cb.EPI_STORE_F32)
    x0 = _rand((M, N), torch.float32, 8)
    x = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32)
    F = N // 2
    packed = Wt[torch.as_tensor(_pack_rows(F), device=DEV)].contiguous()
    act = torch.zeros((M, F), dtype=torch.float32, device=DEV)
    cb.confspec_op_gemm(ctx, A, packed, act, M, N, K, cb.EPI_SWIGLU)
    torch.cuda.synchronize()
    s = np.abs(ref).max()
    assert np.abs(f64(out) - ref).max() <= 1e-5 * s
    assert np.abs(f64(x) - (f64(x0) + ref)).max() <= 1e-5 * max(s, 4.0)
    ref_act = O.silu(ref[:, :F]) * ref[:, F:]
    assert np.abs(f64(act) - ref_act).max() <= 1e-5 * np.abs(ref_act).max()
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("dtype,d", [("bf16", 1536), ("fp32", 256), ("bf16", 5120), ("bf16", 6400)])
def test_rmsnorm(dtype, d):
    print(f"rmsnorm {dtype} d={d}", flush=True)
    ctx, base = _ctx(dtype, d_model=d, head_dim=128 if dtype == "bf16" else 64, n_kv_heads=2 if dtype == "bf16" else 4)
    td = W.torch_dtype(dtype)
    x = _rand((37, d), torch.float32, 9, 3.0)
    g = (1 + 0.1 * _rand((d,), torch.float32, 10)).to(td)
    out = torch.zeros((37, d), dtype=td, device=DEV)
    cb.confspec_op_rmsnorm(ctx, x, g, out, 37)
    torch.cuda.synchronize()
    ref = O.rmsnorm(f64(x), f64(g), base["rms_eps"])
    tol = 2.0 ** -8 if dtype == "bf16" else 1e-6
    assert np.all(np.abs(f64(out) - ref) <= tol * np.abs(ref) + 1e-6)
    cb.confspec_destroy(ctx)


def _batch_structs(wl, batch_dev):
    bs, keep = cb.make_batch(batch_dev.suffix_ids, batch_dev.cu_suffix, batch_dev.prefix_lens,
                             batch_dev.h_cu_suffix, batch_dev.h_prefix_lens)
    return bs, keep


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_rope_split_positions_reach_tens_of_thousands(dtype):
    print(f"rope_split {dtype}", flush=True)
    hd = 128 if dtype == "bf16" else 64
    wl = W.tiny_workload("rope", 3, dtype=dtype, n_q_heads=4, n_kv_heads=2, head_dim=hd, d_model=256,
                         prefix_lens=(16383, 0, 700), suffix_lens=(5, 3, 9), block_size=16)
    m = wl.model
    ctx, _ = _ctx(dtype, head_dim=hd)
    batch = W.make_batch(wl, DEV)
    bs, keep = _batch_structs(wl, batch)
    T = wl.T
    heads = m.n_q_heads + 2 * m.n_kv_heads
    qkv = _rand((T, heads * hd), torch.float32, 11)
    td = W.torch_dtype(dtype)
    q = torch.zeros((T, m.n_q_heads, hd), dtype=td, device=DEV)
    k = torch.zeros((T, m.n_kv_heads, hd), dtype=td, device=DEV)
    v = torch.zeros((T, m.n_kv_heads, hd), dtype=td, device=DEV)
    ws = torch.empty(cb.confspec_workspace_bytes(ctx, T, wl.B), dtype=torch.uint8, device=DEV)
    cb.confspec_op_rope_split(ctx, bs, 16384, qkv, q, k, v, ws)
    torch.cuda.synchronize()
    a = f64(qkv).reshape(T, heads, hd)
    pos = np.concatenate([L + np.arange(S) for L, S in zip(wl.prefix_lens, wl.suffix_lens)])
    rq = O.rope(a[:, :m.n_q_heads], pos, m.rope_theta)
    rk = O.rope(a[:, m.n_q_heads:m.n_q_heads + m.n_kv_heads], pos, m.rope_theta)
    rv = a[:, m.n_q_heads + m.n_kv_heads:]
    tol = 2.0 ** -8 if dtype == "bf16" else 2e-6
    for got, ref in ((q, rq), (k, rk), (v, rv)):
        assert np.abs(f64(got) - ref).max() <= tol * np.abs(ref).max()
    cb.confspec_destroy(ctx)


def _perm_head_rows(n_heads):
    """Row order of wqkv_perm: inside every 128-row head the 32-row blocks go 0, 2, 1, 3."""
    p = np.arange(n_heads * 128)
    blk = (p % 128) // 32
    return np.where(blk == 1, p + 32, np.where(blk == 2, p - 32, p))


@pytest.mark.parametrize("a_terms", [1, 3])
def test_qkv_projection_many_rows_last_round_cut_off(a_terms):
    """8448 rows x 2048 columns are 264 tiles of 256 x 256: one full round and a last column of 33 tiles, which the
    launcher hands to a second launch with 128 x 128 tiles; every element against the oracle's projection + rope."""
    print(f"qkv + rope fused, 8448 rows, a_terms={a_terms}", flush=True)
    hd, d = 128, 256
    wl = W.tiny_workload("qkvwide", 33, dtype="bf16", n_q_heads=12, n_kv_heads=2, head_dim=hd, d_model=d,
                         prefix_lens=tuple(100 * i for i in range(33)), suffix_lens=(256,) * 33, block_size=16)
    m = wl.model
    ctx, _ = _ctx("bf16", head_dim=hd, d_model=d, n_q_heads=12, n_kv_heads=2)
    batch = W.make_batch(wl, DEV)
    bs, keep = _batch_structs(wl, batch)
    T = wl.T
    assert T == 8448
    heads = m.n_q_heads + 2 * m.n_kv_heads
    full = _rand((T, d), torch.float32, 41)
    Wn = _rand((heads * hd, d), torch.float32, 42, 0.1)
    dt = torch.float16 if a_terms == 3 else torch.bfloat16
    h, Wt = full.to(dt), Wn.to(dt)
    Wp = Wt[torch.as_tensor(_perm_head_rows(heads), device=DEV)].contiguous()
    bf = torch.bfloat16
    q = torch.zeros((T + 1, m.n_q_heads, hd), dtype=bf, device=DEV)
    k = torch.zeros((T + 1, m.n_kv_heads, hd), dtype=bf, device=DEV)
    v = torch.zeros((T + 1, m.n_kv_heads, hd), dtype=bf, device=DEV)
    ws = torch.empty(cb.confspec_workspace_bytes(ctx, T, wl.B), dtype=torch.uint8, device=DEV)
    cb.confspec_op_qkv_rope(ctx, bs, 4096, h, a_terms, Wp, q, k, v, ws)
    torch.cuda.synchronize()
    a = (f64(h) @ f64(Wt).T).reshape(T, heads, hd)
    pos = np.concatenate([L + np.arange(S) for L, S in zip(wl.prefix_lens, wl.suffix_lens)])
    rq = O.rope(a[:, :m.n_q_heads], pos, m.rope_theta)
    rk = O.rope(a[:, m.n_q_heads:m.n_q_heads + m.n_kv_heads], pos, m.rope_theta)
    rv = a[:, m.n_q_heads + m.n_kv_heads:]
    for got, ref in ((q, rq), (k, rk), (v, rv)):
        assert np.abs(f64(got[:T]) - ref).max() <= (2.0 ** -8 + 2e-5) * np.abs(ref).max()
        assert torch.all(got[T] == 0)
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("a_terms,with_lo", [(1, False), (3, False), (2, True)])
@pytest.mark.parametrize("suffix_lens", [(5, 3, 9), (200, 77, 130)])
@pytest.mark.parametrize("d", [256, 1024])      # 1024: enough k-tiles for the split-K path at these row counts
def test_qkv_projection_with_rotary_epilogue(a_terms, with_lo, suffix_lens, d):
    print(f"qkv + rope fused a_terms={a_terms} lo={with_lo} S={suffix_lens} d={d}", flush=True)
    hd = 128
    wl = W.tiny_workload("qkvrope", 4, dtype="bf16", n_q_heads=4, n_kv_heads=2, head_dim=hd, d_model=d,
                         prefix_lens=(16383, 0, 700), suffix_lens=suffix_lens, block_size=16)
    m = wl.model
    ctx, _ = _ctx("bf16", head_dim=hd, d_model=d)
    batch = W.make_batch(wl, DEV)
    bs, keep = _batch_structs(wl, batch)
    T = wl.T
    heads = m.n_q_heads + 2 * m.n_kv_heads
    full = _rand((T, d), torch.float32, 31)
    Wn = _rand((heads * hd, d), torch.float32, 32, 0.1)
    if a_terms == 3:
        h = full.to(torch.float16); h64 = f64(h)
        Wt = Wn.to(torch.float16)
    elif a_terms == 2:
        hi = full.to(torch.bfloat16); lo = (full - hi.float()).to(torch.bfloat16)
        h = torch.cat([hi, lo], dim=1).contiguous(); h64 = f64(hi) + f64(lo)
        Wt = Wn.to(torch.bfloat16)
    else:
        h = full.to(torch.bfloat16); h64 = f64(h)
        Wt = Wn.to(torch.bfloat16)
    Wp = Wt[torch.as_tensor(_perm_head_rows(heads), device=DEV)].contiguous()
    bf = torch.bfloat16
    q = torch.zeros((T + 1, m.n_q_heads, hd), dtype=bf, device=DEV)
    k = torch.zeros((T + 1, m.n_kv_heads, hd), dtype=bf, device=DEV)
    v = torch.zeros((T + 1, m.n_kv_heads, hd), dtype=bf, device=DEV)
    los = [torch.zeros_like(t) for t in (q, k, v)] if with_lo else [None, None, None]
    ws = torch.empty(cb.confspec_workspace_bytes(ctx, T, wl.B), dtype=torch.uint8, device=DEV)
    cb.confspec_op_qkv_rope(ctx, bs, 16384, h, a_terms, Wp, q, k, v, ws, q_lo=los[0], k_lo=los[1], v_lo=los[2])
    torch.cuda.synchronize()
    a = (h64 @ f64(Wt).T).reshape(T, heads, hd)
    pos = np.concatenate([L + np.arange(S) for L, S in zip(wl.prefix_lens, wl.suffix_lens)])
    rq = O.rope(a[:, :m.n_q_heads], pos, m.rope_theta)
    rk = O.rope(a[:, m.n_q_heads:m.n_q_heads + m.n_kv_heads], pos, m.rope_theta)
    rv = a[:, m.n_q_heads + m.n_kv_heads:]
    for got, lo_t, ref in ((q, los[0], rq), (k, los[1], rk), (v, los[2], rv)):
        val = f64(got[:T]) + (f64(lo_t[:T]) if with_lo else 0.0)
        tol = 2.0 ** -15 if with_lo else 2.0 ** -8
        assert np.abs(val - ref).max() <= tol * np.abs(ref).max() + 2e-5 * np.abs(ref).max()
        assert torch.all(got[T] == 0)
    cb.confspec_destroy(ctx)


def _attention_case(dtype, hq, hkv, hd, prefix_lens, suffix_lens, block_size=16, seed=20, out_terms=1,
                    precise=False):
    wl = W.tiny_workload("attn", seed, dtype=dtype, n_layers=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd,
                         d_model=256, prefix_lens=prefix_lens, suffix_lens=suffix_lens, block_size=block_size)
    m = wl.model
    ctx, _ = _ctx(dtype, n_layers=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd)
    batch = W.make_batch(wl, DEV)
    kv = W.make_seeded_kv(wl, batch, DEV)
    td = W.torch_dtype(dtype)
    T = wl.T
    lo = {}
    if precise:     # two-term operands: hi = bf16(x), lo = bf16(x - hi); the oracle sees hi + lo
        full = dict(q=_rand((T, hq, hd), torch.float32, seed + 1), k=_rand((T, hkv, hd), torch.float32, seed + 2, 0.5),
                    v=_rand((T, hkv, hd), torch.float32, seed + 3, 0.5))
        hi = {n: x.to(td) for n, x in full.items()}
        lo = {n: (full[n] - hi[n].float()).to(td) for n in full}
        q, ks, vs = hi["q"], hi["k"], hi["v"]
    else:
        q = _rand((T, hq, hd), td, seed + 1)
        ks = _rand((T, hkv, hd), td, seed + 2, 0.5)
        vs = _rand((T, hkv, hd), td, seed + 3, 0.5)
    out = torch.zeros((T, (2 if out_terms == 2 else 1) * hq * hd), dtype=td, device=DEV)
    kvs = cb.make_kv(kv.k_pages, kv.v_pages, batch.block_table, batch.n_blocks, block_size, batch.max_blocks_per_seq)
    bs, keep = _batch_structs(wl, batch)
    ws = torch.empty(cb.confspec_workspace_bytes(ctx, T, wl.B), dtype=torch.uint8, device=DEV)
    layer = 1
    cb.confspec_op_attention(ctx, kvs, bs, layer, q, ks, vs, out, ws, out_terms=out_terms, q_lo=lo.get("q"),
                             k_lo=lo.get("k"), v_lo=lo.get("v"))
    qo = f64(q) + (f64(lo["q"]) if precise else 0.0)
    ko = f64(ks) + (f64(lo["k"]) if precise else 0.0)
    vo = f64(vs) + (f64(lo["v"]) if precise else 0.0)
    torch.cuda.synchronize()
    view = W.OracleKVView(kv, batch)
    got = f64(out.view(torch.float16)) if out_terms == 3 else f64(out)
    if out_terms == 2:
        got = got[:, :hq * hd] + got[:, hq * hd:]
    got = got.reshape(T, hq, hd)
    worst = 0.0
    for b, (L, S) in enumerate(zip(prefix_lens, suffix_lens)):
        lo0 = int(batch.h_cu_suffix[b])
        nblk = (L + block_size - 1) // block_size
        ids = batch.block_table[b, :nblk].cpu().numpy()
        if L:
            kp = O.gather_prefix(view.k_blocks(layer, ids), L)
            vp = O.gather_prefix(view.v_blocks(layer, ids), L)
        else:
            kp = vp = np.zeros((0, hkv, hd))
        k_all = np.concatenate([kp, ko[lo0:lo0 + S]])
        v_all = np.concatenate([vp, vo[lo0:lo0 + S]])
        ref = O.attention(qo[lo0:lo0 + S], k_all, v_all, L)
        worst = max(worst, np.abs(got[lo0:lo0 + S] - ref).max())
    cb.confspec_destroy(ctx)
    return worst


@pytest.mark.parametrize("prefix_lens,suffix_lens", [
    ((128,) * 3, (32,) * 3),                 # whole chunks
    ((0, 5, 77, 200, 1), (1, 7, 33, 64, 100)),   # ragged: empty prefix, page tails, chunk straddling
    ((1000, 17), (96, 130)),                 # several q tiles per trace, long prefix
])
def test_attention_fp32(prefix_lens, suffix_lens):
    print(f"attention fp32 L={prefix_lens} S={suffix_lens}", flush=True)
    err = _attention_case("fp32", 4, 4, 64, prefix_lens, suffix_lens)
    assert err <= 2e-5
    err = _attention_case("fp32", 4, 2, 128, prefix_lens, suffix_lens, block_size=8)
    assert err <= 2e-5


@pytest.mark.parametrize("hq,hkv", [(12, 2), (5, 1), (4, 4)])
@pytest.mark.parametrize("prefix_lens,suffix_lens", [
    ((128,) * 3, (32,) * 3),
    ((0, 5, 77, 200, 1), (1, 7, 33, 64, 100)),
    ((1000, 17), (96, 130)),
])
def test_attention_bf16(hq, hkv, prefix_lens, suffix_lens):
    print(f"attention bf16 hq={hq} hkv={hkv} L={prefix_lens} S={suffix_lens}", flush=True)
    err = _attention_case("bf16", hq, hkv, 128, prefix_lens, suffix_lens)
    print("  max abs err", err, flush=True)
    assert err <= 6e-3


def test_attention_bf16_two_term_output():
    print("attention bf16 two-term output", flush=True)
    plain = _attention_case("bf16", 12, 2, 128, (300, 17), (96, 130))
    two = _attention_case("bf16", 12, 2, 128, (300, 17), (96, 130), out_terms=2)
    print("  plain", plain, "two-term", two, flush=True)
    assert two <= plain and two <= 6e-3


@pytest.mark.parametrize("prefix_lens,suffix_lens", [((300, 17, 0), (96, 130, 5)), ((64, 2049), (64, 33))])
def test_attention_bf16_two_term_operands(prefix_lens, suffix_lens):
    """q, suffix k / v and the probabilities as hi + lo pairs: the result must track the fp64 attention
    of the 16-bit-mantissa operands far more closely than a single bf16 rounding allows."""
    print(f"attention bf16 precise L={prefix_lens} S={suffix_lens}", flush=True)
    err = _attention_case("bf16", 12, 2, 128, prefix_lens, suffix_lens, out_terms=2, precise=True)
    print("  max abs err", err, flush=True)
    assert err <= 2e-4
    err5 = _attention_case("bf16", 5, 1, 128, prefix_lens, suffix_lens, out_terms=2, precise=True)
    assert err5 <= 2e-4


@pytest.mark.parametrize("split", [0, 2, 3, 4, 5])
def test_attention_bf16_split_kv_merge_matches_unsplit(split):
    """Force many key-range pieces (planner's choice, equal pieces, front-loaded pieces): the merged
    result must meet the same bound as the unsplit one."""
    print(f"attention bf16 forced splits, mode {split}", flush=True)
    cb.confspec_tune(None, "attn_min_chunks", 1)
    cb.confspec_tune(None, "attn_target_items", 1024)
    cb.confspec_tune(None, "attn_split", split)
    try:
        err = _attention_case("bf16", 12, 2, 128, (700, 64, 0, 3000), (40, 96, 20, 7))
        err2 = _attention_case("bf16", 12, 2, 128, (700, 64, 0, 3000), (40, 96, 20, 7), out_terms=2)
        err3 = _attention_case("bf16", 8, 8, 128, (130, 2500, 17, 900, 64, 1, 333, 1200, 5), (33, 5, 129, 64, 1, 200, 16, 77, 250))
        assert err2 <= 6e-3 and err3 <= 6e-3
    finally:
        cb.confspec_tune(None, "attn_min_chunks", 4)
        cb.confspec_tune(None, "attn_target_items", 512)
        cb.confspec_tune(None, "attn_split", 0)
    print("  max abs err", err, flush=True)
    assert err <= 6e-3


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_verdict_head_and_gate(dtype):
    print(f"verdict gate {dtype}", flush=True)
    d, V = 256, 512
    hd = 128 if dtype == "bf16" else 64
    ctx, base = _ctx(dtype, d_model=d, vocab=V, head_dim=hd)
    wl = W.tiny_workload("vg", 31, dtype=dtype, d_model=d, vocab=V, head_dim=hd, n_q_heads=4, n_kv_heads=2,
                         prefix_lens=(3,) * 40, suffix_lens=tuple(1 + (i % 5) for i in range(40)), block_size=16)
    batch = W.make_batch(wl, DEV)
    bs, keep = _batch_structs(wl, batch)
    td = W.torch_dtype(dtype)
    T, B = wl.T, wl.B
    x = _rand((T, d), torch.float32, 32, 2.0)
    g = (1 + 0.1 * _rand((d,), torch.float32, 33)).to(td)
    lm = _rand((V, d), td, 34, 0.08)
    vids, taus = [7, 300, 12], [0.0, 0.4, 0.6, 0.9, 1.0]
    logits = torch.zeros((B, 3), dtype=torch.float32, device=DEV)
    conf = torch.zeros(B, dtype=torch.float32, device=DEV)
    verdict = torch.zeros(B, dtype=torch.int32, device=DEV)
    accept = torch.zeros((5, B), dtype=torch.uint8, device=DEV)
    ws = torch.empty(cb.confspec_workspace_bytes(ctx, T, B), dtype=torch.uint8, device=DEV)
    cb.confspec_op_verdict_gate(ctx, bs, x, g, lm, vids, taus, ws, logits, conf, verdict, accept)
    torch.cuda.synchronize()
    xs, gs, lms = f64(x), f64(g), f64(lm)
    for b in range(B):
        last = int(batch.h_cu_suffix[b + 1]) - 1
        z = O.verdict_logits(xs[last], gs, lms[vids], base["rms_eps"])
        p, r, c = O.confidence(z)
        assert np.abs(f64(logits[b]) - z).max() <= 2e-5 * max(1.0, np.abs(z).max())
        assert abs(float(conf[b]) - c) <= 1e-5
        if np.sort(z)[-1] - np.sort(z)[-2] > 1e-4:
            assert int(verdict[b]) == r
        want = O.gate(np.array([c]), taus)[:, 0]
        for i, t in enumerate(taus):
            if abs(c - t) > 1e-5:
                assert int(accept[i, b]) == int(want[i])
    assert accept[0].all() and accept.cpu().numpy()[:-1].sum() > accept.cpu().numpy()[-1].sum()
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("epi", ["store", "resid", "swiglu"])
def test_gemm_bf16_wide_output_split_into_two_launches(epi):
    """Default tile choice on an output wide enough for 256x256 tiles whose last round of 256 tiles
    would be nearly empty: the trailing columns go to a second launch with 128x128 tiles."""
    print(f"gemm bf16 wide split {epi}", flush=True)
    ctx, _ = _ctx("bf16")
    M, N, K = 700, 256 * 90, 128                      # 3 x 90 tiles of 256: one full round + 14 tiles
    A = _rand((M, K), torch.bfloat16, 11)
    Wt = _rand((N, K), torch.bfloat16, 12, 0.05)
    ref = f64(A) @ f64(Wt).T
    if epi == "swiglu":
        F = N // 2
        out = torch.zeros((M + 2, F), dtype=torch.bfloat16, device=DEV)
        cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, cb.EPI_SWIGLU)
        torch.cuda.synchronize()
        r3 = ref.reshape(M, N // 64, 2, 32)           # packed layout: 32 gate columns, then their 32 up columns
        want = (O.silu(r3[:, :, 0, :]) * r3[:, :, 1, :]).reshape(M, F)
        err = np.abs(f64(out[:M]) - want)
        assert np.all(err <= 2.0 ** -8 * np.abs(want) + 1e-4 * np.abs(want).max())
        assert torch.all(out[M:] == 0)
    else:
        x0 = _rand((M + 2, N), torch.float32, 13)
        x = x0.clone()
        cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32 if epi == "resid" else cb.EPI_STORE_F32)
        torch.cuda.synchronize()
        want = ref + (f64(x0[:M]) if epi == "resid" else 0.0)
        assert np.abs(f64(x[:M]) - want).max() <= 2e-5 * max(np.abs(ref).max(), 4.0)
        assert torch.equal(x[M:], x0[M:])
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("a_terms", [1, 2])
@pytest.mark.parametrize("M", [3072, 2990])
def test_gemm_bf16_default_cut_into_one_tile_per_cu(M, a_terms):
    """A little more than 256 tiles of 128x128 that are at most 256 tiles of 192x96: the default choice takes the
    latter (residual and store epilogues)."""
    print(f"gemm bf16 192x96 cut M={M} a_terms={a_terms}", flush=True)
    ctx, _ = _ctx("bf16")
    N, K = 1536, 320
    full = _rand((M, K), torch.float32, 61)
    if a_terms == 2:
        hi = full.to(torch.bfloat16)
        lo = (full - hi.float()).to(torch.bfloat16)
        A = torch.cat([hi, lo], dim=1).contiguous()
        a64 = f64(hi) + f64(lo)
    else:
        A = full.to(torch.bfloat16)
        a64 = f64(A)
    Wt = _rand((N, K), torch.bfloat16, 62, 0.05)
    ref = a64 @ f64(Wt).T
    x0 = _rand((M + 2, N), torch.float32, 63)
    x = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32, a_terms=a_terms)
    torch.cuda.synchronize()
    assert np.abs(f64(x[:M]) - (ref + f64(x0[:M]))).max() <= 2e-5 * max(np.abs(ref).max(), 4.0)
    assert torch.equal(x[M:], x0[M:])
    out = torch.full((M + 2, N), 7.0, dtype=torch.float32, device=DEV)
    cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, cb.EPI_STORE_F32, a_terms=a_terms)
    torch.cuda.synchronize()
    assert np.abs(f64(out[:M]) - ref).max() <= 2e-5 * np.abs(ref).max()
    assert torch.all(out[M:] == 7.0)
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("M", [1, 32, 128, 300, 1000])
@pytest.mark.parametrize("epi,a_terms", [("store", 1), ("resid", 1), ("swiglu", 1), ("resid", 2), ("swiglu", 2)])
def test_gemm_bf16_split_k_for_short_outputs(M, epi, a_terms):
    """Outputs of few tiles, with scratch: k slices as separate workgroups, added in a fixed order."""
    print(f"gemm bf16 split-K M={M} {epi} a_terms={a_terms}", flush=True)
    ctx, _ = _ctx("bf16")
    N, K = 512, 2240                                  # 35 k-tiles: slices of unequal length
    full = _rand((M, K), torch.float32, 21)
    if a_terms == 2:
        hi = full.to(torch.bfloat16)
        lo = (full - hi.float()).to(torch.bfloat16)
        A = torch.cat([hi, lo], dim=1).contiguous()
        a64 = f64(hi) + f64(lo)
    else:
        A = full.to(torch.bfloat16)
        a64 = f64(A)
    Wt = _rand((N, K), torch.bfloat16, 22, 0.05)
    ref = a64 @ f64(Wt).T
    nbytes = cb.confspec_op_gemm_scratch_bytes(ctx, M, N, K, a_terms)
    assert nbytes > 0
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    if epi == "swiglu":
        F = N // 2
        out = torch.zeros((M + 1, F), dtype=torch.bfloat16, device=DEV)
        cb.confspec_op_gemm(ctx, A, Wt, out, M, N, K, cb.EPI_SWIGLU, a_terms=a_terms, scratch=scratch)
        torch.cuda.synchronize()
        r3 = ref.reshape(M, N // 64, 2, 32)
        want = (O.silu(r3[:, :, 0, :]) * r3[:, :, 1, :]).reshape(M, F)
        assert np.all(np.abs(f64(out[:M]) - want) <= 2.0 ** -8 * np.abs(want) + 1e-4 * np.abs(want).max())
        assert torch.all(out[M:] == 0)
        again = torch.zeros_like(out)
        cb.confspec_op_gemm(ctx, A, Wt, again, M, N, K, cb.EPI_SWIGLU, a_terms=a_terms, scratch=scratch)
        torch.cuda.synchronize()
        assert torch.equal(out, again)                # fixed summation order
    else:
        x0 = _rand((M + 1, N), torch.float32, 23)
        x = x0.clone()
        cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32 if epi == "resid" else cb.EPI_STORE_F32,
                            a_terms=a_terms, scratch=scratch)
        torch.cuda.synchronize()
        want = ref + (f64(x0[:M]) if epi == "resid" else 0.0)
        assert np.abs(f64(x[:M]) - want).max() <= 2e-5 * max(np.abs(ref).max(), 4.0)
        assert torch.equal(x[M:], x0[M:])
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("M,N,K,a_terms,slices", [(3072, 1536, 4160, 1, 3), (2900, 1536, 4160, 3, 3), (2048, 2048, 4160, 1, 4),
                                                  (3072, 1536, 2112, 2, 3), (3072, 1536, 1536, 1, 0)])
def test_gemm_bf16_split_k_long_k_big_tiles(M, N, K, a_terms, slices):
    """A long k range over an output of few 256 x 256 tiles: 3..6 k slices of such tiles, then the fixed-order sum.
    `slices` is what the scratch size has to say (0: this shape is not split)."""
    print(f"gemm bf16 big-tile split-K M={M} N={N} K={K} a_terms={a_terms}", flush=True)
    ctx, _ = _ctx("bf16")
    nbytes = cb.confspec_op_gemm_scratch_bytes(ctx, M, N, K, a_terms)
    assert nbytes == slices * M * N * 4
    full = _rand((M, K), torch.float32, 71)
    if a_terms == 2:
        hi = full.to(torch.bfloat16)
        lo = (full - hi.float()).to(torch.bfloat16)
        A = torch.cat([hi, lo], dim=1).contiguous()
        a64 = f64(hi) + f64(lo)
        Wt = _rand((N, K), torch.bfloat16, 72, 0.05)
    elif a_terms == 3:
        A = full.to(torch.float16)
        a64 = f64(A)
        Wt = _rand((N, K), torch.float32, 72, 0.05).to(torch.float16)
    else:
        A = full.to(torch.bfloat16)
        a64 = f64(A)
        Wt = _rand((N, K), torch.bfloat16, 72, 0.05)
    ref = a64 @ f64(Wt).T
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)
    x0 = _rand((M + 1, N), torch.float32, 73)
    x = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32, a_terms=a_terms, scratch=scratch)
    torch.cuda.synchronize()
    assert np.abs(f64(x[:M]) - (ref + f64(x0[:M]))).max() <= 2e-5 * max(np.abs(ref).max(), 4.0)
    assert torch.equal(x[M:], x0[M:])
    again = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, again, M, N, K, cb.EPI_RESID_F32, a_terms=a_terms, scratch=scratch)
    torch.cuda.synchronize()
    assert torch.equal(x, again)                      # fixed summation order
    unsplit = x0.clone()                              # without scratch: one workgroup per tile, the whole k range
    cb.confspec_op_gemm(ctx, A, Wt, unsplit, M, N, K, cb.EPI_RESID_F32, a_terms=a_terms)
    torch.cuda.synchronize()
    assert np.abs(f64(unsplit[:M]) - f64(x[:M])).max() <= 2e-5 * max(np.abs(ref).max(), 4.0)
    cb.confspec_destroy(ctx)


@pytest.mark.parametrize("M,N,K,scratch", [(300, 512, 192, False), (700, 256 * 90, 128, False), (32, 512, 2240, True),
                                           (3072, 1536, 128, False)])   # the last: one 192x96 tile per CU
def test_gemm_fp16_operands_all_epilogues(M, N, K, scratch):
    """Activation format 3: A and W hold IEEE half values, the SwiGLU result is written as half."""
    print(f"gemm fp16 operands M={M} N={N} K={K} scratch={scratch}", flush=True)
    ctx, _ = _ctx("bf16")
    A = _rand((M, K), torch.float32, 51).to(torch.float16)
    Wt = _rand((N, K), torch.float32, 52, 0.05).to(torch.float16)
    ref = f64(A) @ f64(Wt).T
    sc = None
    if scratch:
        sc = torch.empty(cb.confspec_op_gemm_scratch_bytes(ctx, M, N, K, 3), dtype=torch.uint8, device=DEV)
        assert sc.numel() > 0
    x0 = _rand((M + 1, N), torch.float32, 53)
    st = torch.zeros((M + 1, N), dtype=torch.float32, device=DEV)
    x = x0.clone()
    cb.confspec_op_gemm(ctx, A, Wt, st, M, N, K, cb.EPI_STORE_F32, a_terms=3, scratch=sc)
    cb.confspec_op_gemm(ctx, A, Wt, x, M, N, K, cb.EPI_RESID_F32, a_terms=3, scratch=sc)
    F = N // 2
    act = torch.zeros((M + 1, F), dtype=torch.float16, device=DEV)
    cb.confspec_op_gemm(ctx, A, Wt, act, M, N, K, cb.EPI_SWIGLU, a_terms=3, out_terms=3, scratch=sc)
    torch.cuda.synchronize()
    scale = max(np.abs(ref).max(), 4.0)
    assert np.abs(f64(st[:M]) - ref).max() <= 2e-5 * scale and torch.all(st[M:] == 0)
    assert np.abs(f64(x[:M]) - (f64(x0[:M]) + ref)).max() <= 2e-5 * scale and torch.equal(x[M:], x0[M:])
    r3 = ref.reshape(M, N // 64, 2, 32)
    want = (O.silu(r3[:, :, 0, :]) * r3[:, :, 1, :]).reshape(M, F)
    assert np.all(np.abs(f64(act[:M]) - want) <= 2.0 ** -11 * np.abs(want) + 1e-4 * np.abs(want).max())
    assert torch.all(act[M:] == 0)
    cb.confspec_destroy(ctx)


def test_rmsnorm_fp16_output():
    print("rmsnorm fp16 output", flush=True)
    d = 1536
    ctx, base = _ctx("bf16", d_model=d)
    x = _rand((37, d), torch.float32, 9, 3.0)
    g = (1 + 0.1 * _rand((d,), torch.float32, 10)).to(torch.bfloat16)
    out = torch.zeros((38, d), dtype=torch.float16, device=DEV)
    cb.confspec_op_rmsnorm(ctx, x, g, out, 37, out_terms=3)
    torch.cuda.synchronize()
    ref = O.rmsnorm(f64(x), f64(g), base["rms_eps"])
    assert np.all(np.abs(f64(out[:37]) - ref) <= 2.0 ** -11 * np.abs(ref) + 1e-6)
    assert torch.all(out[37] == 0)
    cb.confspec_destroy(ctx)


def test_fp16_stores_saturate_instead_of_overflowing():
    """Activations beyond the half range (gains of about 1e5) are stored as +-65504, never as an infinity: the
    conversion is clamp to the largest finite half, then round to nearest even, which numpy's half conversion
    of the clamped fp64 value reproduces."""
    print("fp16 saturation", flush=True)
    d = 1536
    ctx, base = _ctx("bf16", d_model=d)
    x = _rand((9, d), torch.float32, 91, 3.0)
    g = (1.0e5 * (1 + 0.1 * _rand((d,), torch.float32, 92))).to(torch.bfloat16)
    out = torch.zeros((9, d), dtype=torch.float16, device=DEV)
    cb.confspec_op_rmsnorm(ctx, x, g, out, 9, out_terms=3)
    torch.cuda.synchronize()
    ref = O.rmsnorm(f64(x), f64(g), base["rms_eps"])
    assert np.abs(ref).max() > 2e5 and (np.abs(ref) < 6e4).any()            # both sides of the range occur
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    want = np.clip(ref, -65504.0, 65504.0).astype(np.float16)
    inside = np.abs(ref) < 65000.0
    assert np.array_equal(got[~inside & (np.abs(ref) > 65520.0)], want[~inside & (np.abs(ref) > 65520.0)])
    assert np.all(np.abs(got[inside].astype(np.float64) - ref[inside]) <= 2.0 ** -10 * np.abs(ref[inside]))
    # the SwiGLU epilogue and the split-K reduce: products far beyond the range
    M, F, K = 70, 128, 64
    A = torch.full((M, K), 30.0, dtype=torch.float16, device=DEV)
    Wt = torch.full((2 * F, K), 20.0, dtype=torch.float16, device=DEV)      # gate = up = 38400 -> silu(g) * u ~ 1.5e9
    Wt[::2] *= -1                                                            # negative up values in half of the blocks' rows
    act = torch.zeros((M, F), dtype=torch.float16, device=DEV)
    cb.confspec_op_gemm(ctx, A, Wt, act, M, 2 * F, K, cb.EPI_SWIGLU, a_terms=3, out_terms=3)
    torch.cuda.synchronize()
    a = act.cpu().numpy()
    assert np.isfinite(a).all() and np.abs(a).max() == 65504.0
    cb.confspec_destroy(ctx)


def test_attention_bf16_fp16_output():
    print("attention fp16 output", flush=True)
    err = _attention_case("bf16", 12, 2, 128, (300, 17, 0), (96, 130, 5), out_terms=3)
    assert err <= 6e-3
    cb.confspec_tune(None, "attn_min_chunks", 1)
    cb.confspec_tune(None, "attn_split", 3)
    try:
        err = _attention_case("bf16", 12, 2, 128, (700, 64), (40, 96), out_terms=3)     # through the merge kernel
    finally:
        cb.confspec_tune(None, "attn_min_chunks", 4)
        cb.confspec_tune(None, "attn_split", 0)
    assert err <= 6e-3
