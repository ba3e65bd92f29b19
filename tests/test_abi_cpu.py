"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and rejects bad
arguments before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2602_18447_amd import binding as cb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for hdr in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not hdr.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(confspec_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    declared = _declared_symbols()
    assert {"confspec_create", "confspec_verify", "confspec_pack_weights", "confspec_workspace_bytes",
            "confspec_op_gemm", "confspec_op_attention", "confspec_op_verdict_gate", "confspec_cascade"} <= declared
    for name in declared:
        assert hasattr(cb.lib, name), f"{name} declared in include/ but not exported"
    assert set(cb.EXPORTED) == declared
    assert cb.confspec_version() == "0.1"


def _cfg(dtype="bf16", **kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=512, vocab=1000,
                rope_theta=1e6, rms_eps=1e-6, dtype=dtype)
    base.update(kw)
    return cb.make_model_cfg(**base)


def test_create_rejects_unsupported_shapes():
    for bad in (dict(head_dim=64), dict(n_q_heads=5), dict(d_model=200), dict(d_ffn=100)):
        with pytest.raises(cb.ConfSpecError) as e:
            cb.confspec_create(_cfg(**bad))
        assert e.value.code == cb.E_UNSUPPORTED
    with pytest.raises(cb.ConfSpecError) as e:
        cb.confspec_create(_cfg(vocab=0))
    assert e.value.code == cb.E_INVALID_ARG
    ctx = cb.confspec_create(_cfg("fp32", head_dim=64, n_kv_heads=4))
    cb.confspec_destroy(ctx)


def test_workspace_size_is_monotone_and_aligned():
    ctx = cb.confspec_create(_cfg())
    a = cb.confspec_workspace_bytes(ctx, 64, 2)
    b = cb.confspec_workspace_bytes(ctx, 128, 2)
    c = cb.confspec_workspace_bytes(ctx, 128, 8)
    assert a % 256 == 0 and a < b <= c
    with pytest.raises(cb.ConfSpecError):
        cb.confspec_workspace_bytes(ctx, 0, 1)
    cb.confspec_destroy(ctx)


def _no_gpu_here():
    """The calls below hand made-up addresses to the library and rely on validation stopping them before any launch;
    a mistake in such a test must never reach a real GPU, so they only run where there is none."""
    import torch
    if torch.cuda.device_count() > 0:
        pytest.skip("fake-pointer validation tests run on machines without a GPU only")


class _FakeDev:
    """Stands in for a device tensor: a fixed fake address, never dereferenced because every call in
    this file must fail validation before the first launch."""

    def __init__(self, addr=0x10000, nbytes=1 << 40):
        self._a, self._n = addr, nbytes

    def data_ptr(self):
        return self._a

    def numel(self):
        return self._n

    def element_size(self):
        return 1


def _verify_args(ctx_cfg, B=2, S=(3, 2), L=(5, 0), block_size=16):
    fake = _FakeDev()
    n_layers = ctx_cfg.n_layers
    ptrs = [fake] * n_layers
    w, keep_w = cb.make_weights(fake, fake, fake, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, packed=1)
    kv = cb.make_kv(fake, fake, fake, 8, block_size, 4)
    cu = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    batch, keep_b = cb.make_batch(fake, fake, fake, cu, np.asarray(L, dtype=np.int32))
    return fake, w, kv, batch, (keep_w, keep_b)


def _expect(ctx, code, fn):
    with pytest.raises(cb.ConfSpecError) as e:
        fn()
    assert e.value.code == code, str(e.value)
    assert cb.confspec_last_error(ctx) != ""


def test_verify_validates_before_any_launch():
    _no_gpu_here()
    cfg = _cfg()
    ctx = cb.confspec_create(cfg)
    fake, w, kv, batch, keep = _verify_args(cfg)
    out = (fake, fake, fake, fake)
    ok = dict(verdict_ids=[1, 2], taus=[0.9])

    def call(w=w, kv=kv, batch=batch, ws=fake, out=out, **kw):
        a = dict(ok)
        a.update(kw)
        return cb.confspec_verify(ctx, w, kv, batch, a["verdict_ids"], a["taus"], ws, *out, stream=0)

    _expect(ctx, cb.E_INVALID_ARG, lambda: call(verdict_ids=[1]))
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(verdict_ids=list(range(9))))
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(verdict_ids=[3, 3]))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(verdict_ids=[1, 1000]))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(verdict_ids=[-1, 5]))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(taus=[1.5]))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(taus=[float("nan")]))
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(taus=[]))
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(out=(None, fake, fake, fake)))
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(ws=None))
    _expect(ctx, cb.E_WORKSPACE, lambda: call(ws=_FakeDev(0x10000, 1024)))
    _expect(ctx, cb.E_WORKSPACE, lambda: call(ws=_FakeDev(0x10010)))
    # unpacked weights are refused
    w2, k2 = cb.make_weights(fake, fake, fake, *[[fake] * 2] * 6, packed=0)
    _expect(ctx, cb.E_INVALID_ARG, lambda: call(w=w2))
    # batch problems
    _, _, _, bad, k3 = _verify_args(cfg, S=(3, 0))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(batch=bad))            # empty suffix
    _, _, _, bad, k4 = _verify_args(cfg, L=(65, 0))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(batch=bad))            # prefix longer than the block table
    _, _, _, bad, k5 = _verify_args(cfg, L=(-1, 0))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(batch=bad))
    bad_T = cb.Batch(batch.B, batch.T + 1, batch.suffix_ids, batch.cu_suffix, batch.prefix_lens,
                     batch.h_cu_suffix, batch.h_prefix_lens)
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(batch=bad_T))
    # bf16 attention is written for 16-token pages
    _, _, kv8, _, k6 = _verify_args(cfg, block_size=8)
    _expect(ctx, cb.E_UNSUPPORTED, lambda: call(kv=kv8))
    cb.confspec_destroy(ctx)


def test_shared_context_groups_are_validated():
    _no_gpu_here()
    cfg = _cfg()
    ctx = cb.confspec_create(cfg)
    fake, w, kv, batch, keep = _verify_args(cfg, B=3, L=(32, 32, 16), S=(3, 4, 5))

    def call(gs):
        cb.confspec_verify_shared(ctx, w, kv, batch, fake, np.asarray(gs, dtype=np.int32), [1, 2], [0.9], fake, fake, fake,
                                  fake, fake, stream=0)
    for bad in ([1, 3], [0, 2], [0, 2, 2, 3], [0, 3, 2, 3]):          # not from 0, not to B, not increasing
        _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call(bad))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call([0, 3]))              # prefix lengths 32, 32, 16 in one group
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: call([0, 1, 3]))           # 32 and 16 in the second group
    cb.confspec_destroy(ctx)


def test_op_gemm_and_tune_validation():
    _no_gpu_here()
    ctx = cb.confspec_create(_cfg())
    fake = _FakeDev()
    _expect(ctx, cb.E_UNSUPPORTED, lambda: cb.confspec_op_gemm(ctx, fake, fake, fake, 8, 100, 64, 0, stream=0))
    _expect(ctx, cb.E_UNSUPPORTED, lambda: cb.confspec_op_gemm(ctx, fake, fake, fake, 8, 128, 40, 0, stream=0))
    _expect(ctx, cb.E_INVALID_ARG, lambda: cb.confspec_op_gemm(ctx, fake, fake, fake, 0, 128, 64, 0, stream=0))
    _expect(ctx, cb.E_INVALID_ARG, lambda: cb.confspec_op_gemm(ctx, fake, fake, fake, 8, 128, 64, 7, stream=0))
    for c in (ctx, None):                 # one context's settings, and the defaults of later contexts
        with pytest.raises(cb.ConfSpecError):
            cb.confspec_tune(c, "no_such_key", 1)
        cb.confspec_tune(c, "gemm_tile", 0)
        for bad in (99, 2, 3, 5, 6):      # only the tile shapes that are built
            with pytest.raises(cb.ConfSpecError):
                cb.confspec_tune(c, "gemm_tile", bad)
        cb.confspec_tune(c, "gemm_splitk", 0)
        with pytest.raises(cb.ConfSpecError):
            cb.confspec_tune(c, "gemm_splitk", 65)
    cb.confspec_destroy(ctx)


def test_settings_belong_to_a_context():
    """A setting made on one context leaves another context, and the defaults, alone; a context created after a
    change of the defaults starts from them.  Seen through the packed-weight size, which depends on the number of
    fp16 layers."""
    _no_gpu_here()
    cfg = _cfg(n_layers=8)
    a, b = cb.confspec_create(cfg), cb.confspec_create(cfg)
    base = cb.confspec_packed_bytes(a)
    assert cb.confspec_packed_bytes(b) == base
    cb.confspec_tune(a, "first_layers_f16", 0)
    assert cb.confspec_packed_bytes(a) < base and cb.confspec_packed_bytes(b) == base
    try:
        cb.confspec_tune(None, "split_layers", 2)
        c = cb.confspec_create(cfg)
        assert cb.confspec_packed_bytes(a) < cb.confspec_packed_bytes(c) < base
        assert cb.confspec_packed_bytes(b) == base
        cb.confspec_destroy(c)
    finally:
        cb.confspec_tune(None, "split_layers", -1)
    for ctx in (a, b):
        cb.confspec_destroy(ctx)


def test_cascade_validates_before_any_launch():
    _no_gpu_here()
    cfg_d, cfg_t = _cfg(), _cfg(n_layers=3, d_model=512, n_q_heads=4, d_ffn=1024)
    ctx_d, ctx_t = cb.confspec_create(cfg_d), cb.confspec_create(cfg_t)
    fake, w, kv, batch, keep = _verify_args(cfg_d, B=3, S=(3, 2, 4), L=(5, 0, 7))
    _, w_t, _, _, keep_t = _verify_args(cfg_t, B=3, S=(3, 2, 4), L=(5, 0, 7))
    out = cb.CascadeOut(*([fake.data_ptr()] * 10))
    assert cb.confspec_cascade_scratch_bytes(3, 9, 4) % 256 == 0
    assert cb.confspec_cascade_scratch_bytes(0, 9, 4) == 0

    def call(req=(0, 2, 3), gamma=0.9, ctx_t=ctx_t, out=out, scratch=fake, kv_t=kv, ws_t=fake, parent=None):
        reqs, keep_r = cb.make_requests(fake, np.asarray(req, dtype=np.int32), None if parent is None else fake, parent)
        return cb.confspec_cascade(ctx_d, w, kv, fake, ctx_t, w_t, kv_t, ws_t, batch, reqs, [1, 2], gamma, scratch, out,
                                   stream=0)

    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(req=(0, 2, 2, 3)))      # a request without steps
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(req=(0, 2)))            # does not cover the batch
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(req=(1, 3)))
    _expect(ctx_d, cb.E_INVALID_ARG, lambda: call(req=(0, 1, 2, 3, 4)))    # more requests than traces
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(parent=[-1, 1, -1]))   # a trace cannot continue itself
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(parent=[-1, 0, 1]))    # nor a trace of another request
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(parent=[-2, 0, -1]))
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(gamma=-0.1))
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(gamma=float("nan")))
    _expect(ctx_d, cb.E_INVALID_ARG, lambda: call(ctx_t=None))
    _expect(ctx_d, cb.E_INVALID_ARG, lambda: call(out=cb.CascadeOut()))
    _expect(ctx_d, cb.E_WORKSPACE, lambda: call(scratch=_FakeDev(nbytes=256)))
    _expect(ctx_d, cb.E_WORKSPACE, lambda: call(ws_t=_FakeDev(nbytes=1024)))
    _expect(ctx_d, cb.E_WORKSPACE, lambda: call(scratch=_FakeDev(addr=0x10010)))
    _expect(ctx_d, cb.E_UNSUPPORTED, lambda: call(kv_t=cb.make_kv(fake, fake, fake, 8, 32, 4)))
    ctx_v = cb.confspec_create(_cfg(vocab=2))      # verdict id 2 is outside the large model's vocabulary
    _expect(ctx_d, cb.E_OUT_OF_RANGE, lambda: call(ctx_t=ctx_v))
    for c in (ctx_d, ctx_t, ctx_v):
        cb.confspec_destroy(c)


def test_append_and_generate_validate_before_any_launch():
    _no_gpu_here()
    cfg = _cfg()
    ctx = cb.confspec_create(cfg)
    fake, w, kv, batch, keep = _verify_args(cfg, B=2, S=(3, 2), L=(5, 0))
    out = (fake, fake, fake, fake)

    def append(n, dev=fake):
        return cb.confspec_verify_append(ctx, w, kv, batch, dev, None if n is None else np.asarray(n, dtype=np.int32),
                                         [1, 2], [0.9], fake, *out, stream=0)

    _expect(ctx, cb.E_INVALID_ARG, lambda: append(None))
    _expect(ctx, cb.E_INVALID_ARG, lambda: append([1, 1], dev=None))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: append([4, 0]))              # more than the suffix holds
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: append([0, -1]))
    kv_small = cb.make_kv(fake, fake, fake, 8, 16, 1)                    # 16 rows per trace at most
    batch_full, keep_full = cb.make_batch(fake, fake, fake, np.array([0, 3, 5], dtype=np.int32), np.array([14, 0], dtype=np.int32))
    _expect(ctx, cb.E_OUT_OF_RANGE, lambda: cb.confspec_verify_append(
        ctx, w, kv_small, batch_full, fake, np.array([3, 0], dtype=np.int32), [1, 2], [0.9], fake, *out, stream=0))

    head = cb.HeadOut(fake.data_ptr(), fake.data_ptr(), fake.data_ptr(), None)
    assert cb.confspec_head_scratch_bytes(ctx, 2) % 256 == 0 and cb.confspec_head_scratch_bytes(ctx, 0) == 0
    assert cb.confspec_head_scratch_bytes(ctx, 4) > cb.confspec_head_scratch_bytes(ctx, 2) >= 2 * 1000 * 4

    def gen(head=head, scratch=fake, vids=None, n=None, dev_n=None, ctx=ctx):
        return cb.confspec_generate_step(ctx, w, kv, batch, dev_n, n, vids, fake, scratch, head, stream=0)

    _expect(ctx, cb.E_UNSUPPORTED, gen)                                  # vocab 1000 is not a multiple of 128
    ctx2 = cb.confspec_create(_cfg(vocab=1024))
    _expect(ctx2, cb.E_WORKSPACE, lambda: gen(scratch=_FakeDev(nbytes=1024), ctx=ctx2))
    _expect(ctx2, cb.E_INVALID_ARG, lambda: gen(head=cb.HeadOut(), ctx=ctx2))
    _expect(ctx2, cb.E_INVALID_ARG, lambda: gen(head=cb.HeadOut(*([fake.data_ptr()] * 4)), ctx=ctx2))   # conf_full without verdict ids
    _expect(ctx2, cb.E_INVALID_ARG, lambda: gen(n=np.array([1, 1], dtype=np.int32), ctx=ctx2))          # host counts without device counts
    _expect(ctx2, cb.E_OUT_OF_RANGE, lambda: gen(vids=[1, 5000], ctx=ctx2))
    cb.confspec_destroy(ctx)
    cb.confspec_destroy(ctx2)
