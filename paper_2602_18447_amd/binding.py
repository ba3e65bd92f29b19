"""ctypes binding of libconfspec.so: argument marshalling only.

Every function mirrors the C entry point of the same name (include/confspec.h,
include/confspec_ops.h).  Torch appears only as the owner of device memory and
of the stream handle; every step of the pass runs in the library's kernels.
There is no CPU fallback: if the shared library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CONFSPEC_LIB_PATH") or os.path.join(PKG_DIR, "libconfspec.so")

OK, E_INVALID_ARG, E_UNSUPPORTED, E_WORKSPACE, E_OUT_OF_RANGE, E_HIP = 0, -1, -2, -3, -4, -5
DTYPE_FP32, DTYPE_BF16 = 0, 1
EPI_STORE_F32, EPI_RESID_F32, EPI_SWIGLU = 0, 1, 2
ERROR_NAMES = {OK: "OK", E_INVALID_ARG: "INVALID_ARG", E_UNSUPPORTED: "UNSUPPORTED", E_WORKSPACE: "WORKSPACE",
               E_OUT_OF_RANGE: "OUT_OF_RANGE", E_HIP: "HIP"}


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("mlp_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p)), ("packed", C.c_int32),
                ("n_f16_layers", C.c_int32), ("wqkv_perm", C.POINTER(C.c_void_p)),
                ("wqkv_f16", C.POINTER(C.c_void_p)), ("wo_f16", C.POINTER(C.c_void_p)),
                ("w_gate_up_f16", C.POINTER(C.c_void_p)), ("w_down_f16", C.POINTER(C.c_void_p))]


class KV(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("n_blocks", C.c_int32),
                ("block_size", C.c_int32), ("block_table", C.c_void_p), ("max_blocks_per_seq", C.c_int32)]


class Batch(C.Structure):
    _fields_ = [("B", C.c_int32), ("T", C.c_int32), ("suffix_ids", C.c_void_p), ("cu_suffix", C.c_void_p),
                ("prefix_lens", C.c_void_p), ("h_cu_suffix", C.POINTER(C.c_int32)),
                ("h_prefix_lens", C.POINTER(C.c_int32))]


class Requests(C.Structure):
    _fields_ = [("n_requests", C.c_int32), ("req_start", C.c_void_p), ("h_req_start", C.POINTER(C.c_int32)),
                ("parent", C.c_void_p), ("h_parent", C.POINTER(C.c_int32))]


class CascadeOut(C.Structure):
    _fields_ = [("conf_draft", C.c_void_p), ("verdict_draft", C.c_void_p), ("conf_target", C.c_void_p),
                ("verdict_target", C.c_void_p), ("decision", C.c_void_p), ("escalated", C.c_void_p),
                ("target_ran", C.c_void_p), ("accepted_steps", C.c_void_p), ("selected", C.c_void_p),
                ("conf_used", C.c_void_p)]


class HeadOut(C.Structure):
    _fields_ = [("token", C.c_void_p), ("max_logit", C.c_void_p), ("lse", C.c_void_p), ("conf_full", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    # torch first: it brings its own HIP runtime, and the library must bind to that same copy so that
    # device pointers and streams handed over from torch tensors belong to the runtime that launches.
    import torch  # noqa: F401

    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.confspec_version.restype = C.c_char_p
    lib.confspec_version.argtypes = []
    lib.confspec_create.restype = C.c_int
    lib.confspec_create.argtypes = [P(ModelCfg), C.c_int, P(vp)]
    lib.confspec_destroy.restype = None
    lib.confspec_destroy.argtypes = [vp]
    lib.confspec_last_error.restype = C.c_char_p
    lib.confspec_last_error.argtypes = [vp]
    lib.confspec_workspace_bytes.restype = C.c_int
    lib.confspec_workspace_bytes.argtypes = [vp, i32, i32, C.c_int64, P(sz)]
    lib.confspec_packed_bytes.restype = C.c_int
    lib.confspec_packed_bytes.argtypes = [vp, P(sz)]
    lib.confspec_pack_weights.restype = C.c_int
    lib.confspec_pack_weights.argtypes = [vp, P(Weights), vp, sz, P(vp), P(Weights), vp]
    lib.confspec_verify.restype = C.c_int
    lib.confspec_verify.argtypes = [vp, P(Weights), P(KV), P(Batch), P(i32), i32, P(C.c_float), i32, vp, sz,
                                    vp, vp, vp, vp, vp]
    lib.confspec_op_gemm.restype = C.c_int
    lib.confspec_op_gemm.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.confspec_op_gemm_scratch_bytes.restype = sz
    lib.confspec_op_gemm_scratch_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.confspec_op_rmsnorm.restype = C.c_int
    lib.confspec_op_rmsnorm.argtypes = [vp, vp, vp, vp, i32, i32, vp]
    lib.confspec_op_rope_split.restype = C.c_int
    lib.confspec_op_rope_split.argtypes = [vp, P(Batch), i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.confspec_op_qkv_rope.restype = C.c_int
    lib.confspec_op_qkv_rope.argtypes = [vp, P(Batch), i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.confspec_op_attention.restype = C.c_int
    lib.confspec_op_attention.argtypes = [vp, P(KV), P(Batch), i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.confspec_op_verdict_gate.restype = C.c_int
    lib.confspec_op_verdict_gate.argtypes = [vp, P(Batch), vp, vp, vp, P(i32), i32, P(C.c_float), i32, vp, sz,
                                             vp, vp, vp, vp, vp]
    lib.confspec_verify_append.restype = C.c_int
    lib.confspec_verify_append.argtypes = [vp, P(Weights), P(KV), P(Batch), vp, P(i32), P(i32), i32, P(C.c_float), i32,
                                           vp, sz, vp, vp, vp, vp, vp]
    lib.confspec_head_scratch_bytes.restype = sz
    lib.confspec_head_scratch_bytes.argtypes = [vp, i32]
    lib.confspec_generate_step.restype = C.c_int
    lib.confspec_generate_step.argtypes = [vp, P(Weights), P(KV), P(Batch), vp, P(i32), P(i32), i32, vp, sz, vp, sz,
                                           P(HeadOut), vp]
    lib.confspec_cascade_scratch_bytes.restype = sz
    lib.confspec_cascade_scratch_bytes.argtypes = [i32, i32, i32]
    lib.confspec_cascade.restype = C.c_int
    lib.confspec_cascade.argtypes = [vp, P(Weights), P(KV), vp, sz, vp, P(Weights), P(KV), vp, sz, P(Batch), P(Requests),
                                     P(i32), i32, C.c_float, vp, sz, P(CascadeOut), P(i32), vp]
    lib.confspec_static_scratch_need.restype = C.c_int
    lib.confspec_static_scratch_need.argtypes = [vp, P(Batch), P(sz)]
    lib.confspec_verify_static.restype = C.c_int
    lib.confspec_verify_static.argtypes = [vp, P(Weights), P(KV), P(Batch), P(i32), i32, P(C.c_float), i32,
                                           vp, vp, vp, vp, vp]
    lib.confspec_verify_shared.restype = C.c_int
    lib.confspec_verify_shared.argtypes = [vp, P(Weights), P(KV), P(Batch), vp, P(i32), i32, P(i32), i32, P(C.c_float), i32,
                                           vp, sz, vp, vp, vp, vp, vp]
    lib.confspec_op_workspace_slices.restype = C.c_int
    lib.confspec_op_workspace_slices.argtypes = [vp, i32, i32, P(Batch), P(sz), P(sz), P(i32), P(sz)]
    lib.confspec_phase_timing.restype = C.c_int
    lib.confspec_phase_timing.argtypes = [vp, i32]
    lib.confspec_phase_times.restype = C.c_int
    lib.confspec_phase_times.argtypes = [vp, P(C.c_float), P(i32)]
    lib.confspec_tune.restype = C.c_int
    lib.confspec_tune.argtypes = [vp, C.c_char_p, i32]
    return lib


lib = _load()

EXPORTED = ["confspec_version", "confspec_create", "confspec_destroy", "confspec_last_error",
            "confspec_workspace_bytes", "confspec_packed_bytes", "confspec_pack_weights", "confspec_verify",
            "confspec_op_gemm", "confspec_op_gemm_scratch_bytes", "confspec_op_rmsnorm", "confspec_op_rope_split", "confspec_op_qkv_rope", "confspec_op_attention",
            "confspec_op_verdict_gate", "confspec_tune", "confspec_cascade_scratch_bytes",
            "confspec_cascade", "confspec_verify_append", "confspec_head_scratch_bytes", "confspec_generate_step",
            "confspec_static_scratch_need", "confspec_verify_static", "confspec_phase_timing", "confspec_phase_times", "confspec_verify_shared", "confspec_op_workspace_slices"]


class ConfSpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"confspec error {ERROR_NAMES.get(code, code)}: {msg}")
        self.code = code


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, None for None."""
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = getattr(stream, "cuda_stream", stream)
    return h if h else None


def _check(ctx, rc: int):
    if rc != OK:
        msg = lib.confspec_last_error(ctx).decode() if ctx else ""
        raise ConfSpecError(rc, msg)


# --------------------------------------------------------------------------- #
# thin wrappers, one per C entry point
# --------------------------------------------------------------------------- #
def confspec_version() -> str:
    return lib.confspec_version().decode()


def confspec_create(cfg: ModelCfg, device: int = 0) -> C.c_void_p:
    out = C.c_void_p()
    rc = lib.confspec_create(C.byref(cfg), device, C.byref(out))
    if rc != OK:
        raise ConfSpecError(rc, "confspec_create rejected the model configuration")
    return out


def confspec_destroy(ctx) -> None:
    lib.confspec_destroy(ctx)


def confspec_last_error(ctx) -> str:
    return lib.confspec_last_error(ctx).decode()


def confspec_workspace_bytes(ctx, max_T: int, max_B: int, max_sum_L: int = 0) -> int:
    out = C.c_size_t()
    _check(ctx, lib.confspec_workspace_bytes(ctx, max_T, max_B, max_sum_L, C.byref(out)))
    return out.value


def confspec_packed_bytes(ctx) -> int:
    out = C.c_size_t()
    _check(ctx, lib.confspec_packed_bytes(ctx, C.byref(out)))
    return out.value


def confspec_pack_weights(ctx, w_in: Weights, dev_dst, dst_bytes: int, h_ptr_storage, w_out: Weights,
                          stream=None) -> None:
    _check(ctx, lib.confspec_pack_weights(ctx, C.byref(w_in), _ptr(dev_dst), dst_bytes, h_ptr_storage,
                                          C.byref(w_out), _stream_handle(stream)))


def confspec_verify(ctx, w: Weights, kv: KV, batch: Batch, verdict_ids: Sequence[int], taus: Sequence[float],
                    workspace, logits, conf, verdict, accept, stream=None) -> None:
    nv, nt = len(verdict_ids), len(taus)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    tau = (C.c_float * max(nt, 1))(*[float(t) for t in taus])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(ctx, lib.confspec_verify(ctx, C.byref(w), C.byref(kv), C.byref(batch), ids, nv, tau, nt,
                                    _ptr(workspace), ws_bytes, _ptr(logits), _ptr(conf), _ptr(verdict),
                                    _ptr(accept), _stream_handle(stream)))


def confspec_verify_shared(ctx, w: Weights, kv: KV, batch: Batch, group_start, h_group_start, verdict_ids: Sequence[int],
                           taus: Sequence[float], workspace, logits, conf, verdict, accept, stream=None) -> None:
    """group_start: device int32 tensor [n_groups + 1]; h_group_start: the same values as a host int32 numpy array."""
    import numpy as np
    nv, nt = len(verdict_ids), len(taus)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    tau = (C.c_float * max(nt, 1))(*[float(t) for t in taus])
    hg = np.ascontiguousarray(h_group_start, dtype=np.int32)
    _check(ctx, lib.confspec_verify_shared(ctx, C.byref(w), C.byref(kv), C.byref(batch), _ptr(group_start),
                                           hg.ctypes.data_as(C.POINTER(C.c_int32)), len(hg) - 1, ids, nv, tau, nt,
                                           _ptr(workspace), _nbytes(workspace), _ptr(logits), _ptr(conf), _ptr(verdict),
                                           _ptr(accept), _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 64 << 20


def confspec_static_scratch_need(ctx, batch: Batch) -> int:
    out = C.c_size_t()
    _check(ctx, lib.confspec_static_scratch_need(ctx, C.byref(batch), C.byref(out)))
    return out.value


def confspec_verify_static(ctx, w: Weights, kv: KV, batch: Batch, verdict_ids: Sequence[int], taus: Sequence[float],
                           logits, conf, verdict, accept, stream=None) -> None:
    nv, nt = len(verdict_ids), len(taus)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    tau = (C.c_float * max(nt, 1))(*[float(t) for t in taus])
    _check(ctx, lib.confspec_verify_static(ctx, C.byref(w), C.byref(kv), C.byref(batch), ids, nv, tau, nt,
                                           _ptr(logits), _ptr(conf), _ptr(verdict), _ptr(accept),
                                           _stream_handle(stream)))


def confspec_verify_append(ctx, w: Weights, kv: KV, batch: Batch, n_append, h_n_append, verdict_ids: Sequence[int],
                           taus: Sequence[float], workspace, logits, conf, verdict, accept, stream=None) -> None:
    """n_append: device int32 tensor [B]; h_n_append: the same counts as a host int32 numpy array."""
    import numpy as np
    nv, nt = len(verdict_ids), len(taus)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    tau = (C.c_float * max(nt, 1))(*[float(t) for t in taus])
    hn = None if h_n_append is None else np.ascontiguousarray(h_n_append, dtype=np.int32)
    hp = None if hn is None else hn.ctypes.data_as(C.POINTER(C.c_int32))
    _check(ctx, lib.confspec_verify_append(ctx, C.byref(w), C.byref(kv), C.byref(batch), _ptr(n_append), hp, ids, nv,
                                           tau, nt, _ptr(workspace), _nbytes(workspace), _ptr(logits), _ptr(conf),
                                           _ptr(verdict), _ptr(accept), _stream_handle(stream)))


def confspec_head_scratch_bytes(ctx, max_B: int) -> int:
    return int(lib.confspec_head_scratch_bytes(ctx, max_B))


def confspec_generate_step(ctx, w: Weights, kv: KV, batch: Batch, n_append, h_n_append, verdict_ids, workspace,
                           head_scratch, out: HeadOut, stream=None) -> None:
    """n_append / h_n_append: device tensor and host int32 array, or both None; verdict_ids: sequence or None."""
    import numpy as np
    nv = 0 if verdict_ids is None else len(verdict_ids)
    ids = None if verdict_ids is None else (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    hn = None if h_n_append is None else np.ascontiguousarray(h_n_append, dtype=np.int32)
    hp = None if hn is None else hn.ctypes.data_as(C.POINTER(C.c_int32))
    _check(ctx, lib.confspec_generate_step(ctx, C.byref(w), C.byref(kv), C.byref(batch), _ptr(n_append), hp, ids, nv,
                                           _ptr(workspace), _nbytes(workspace), _ptr(head_scratch), _nbytes(head_scratch),
                                           C.byref(out), _stream_handle(stream)))


def confspec_op_gemm(ctx, A, W, out, M: int, N: int, K: int, epilogue: int, a_terms: int = 1, out_terms: int = 1,
                     scratch=None, stream=None) -> None:
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(ctx, lib.confspec_op_gemm(ctx, _ptr(A), _ptr(W), _ptr(out), M, N, K, epilogue, a_terms, out_terms,
                                     _ptr(scratch), nbytes, _stream_handle(stream)))


def confspec_op_gemm_scratch_bytes(ctx, M: int, N: int, K: int, a_terms: int = 1) -> int:
    return int(lib.confspec_op_gemm_scratch_bytes(ctx, M, N, K, a_terms))


def confspec_op_rmsnorm(ctx, x, g, out, n_rows: int, out_terms: int = 1, stream=None) -> None:
    _check(ctx, lib.confspec_op_rmsnorm(ctx, _ptr(x), _ptr(g), _ptr(out), n_rows, out_terms,
                                        _stream_handle(stream)))


def confspec_op_rope_split(ctx, batch: Batch, max_prefix_len: int, qkv, q, k, v, workspace, q_lo=None, k_lo=None,
                           v_lo=None, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(ctx, lib.confspec_op_rope_split(ctx, C.byref(batch), max_prefix_len, _ptr(qkv), _ptr(q), _ptr(k), _ptr(v),
                                           _ptr(q_lo), _ptr(k_lo), _ptr(v_lo), _ptr(workspace), ws_bytes,
                                           _stream_handle(stream)))


def confspec_op_qkv_rope(ctx, batch: Batch, max_prefix_len: int, h, a_terms: int, wqkv_perm, q, k, v, workspace,
                         q_lo=None, k_lo=None, v_lo=None, stream=None) -> None:
    _check(ctx, lib.confspec_op_qkv_rope(ctx, C.byref(batch), max_prefix_len, _ptr(h), a_terms, _ptr(wqkv_perm), _ptr(q),
                                         _ptr(k), _ptr(v), _ptr(q_lo), _ptr(k_lo), _ptr(v_lo), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def confspec_op_attention(ctx, kv: KV, batch: Batch, layer: int, q, k_suffix, v_suffix, out, workspace,
                          out_terms: int = 1, q_lo=None, k_lo=None, v_lo=None, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(ctx, lib.confspec_op_attention(ctx, C.byref(kv), C.byref(batch), layer, _ptr(q), _ptr(k_suffix),
                                          _ptr(v_suffix), _ptr(q_lo), _ptr(k_lo), _ptr(v_lo), _ptr(out), out_terms,
                                          _ptr(workspace), ws_bytes, _stream_handle(stream)))


def confspec_op_verdict_gate(ctx, batch: Batch, x, final_norm, lm_head, verdict_ids, taus, workspace, logits, conf,
                             verdict, accept, stream=None) -> None:
    nv, nt = len(verdict_ids), len(taus)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    tau = (C.c_float * max(nt, 1))(*[float(t) for t in taus])
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(ctx, lib.confspec_op_verdict_gate(ctx, C.byref(batch), _ptr(x), _ptr(final_norm), _ptr(lm_head), ids, nv,
                                             tau, nt, _ptr(workspace), ws_bytes, _ptr(logits), _ptr(conf),
                                             _ptr(verdict), _ptr(accept), _stream_handle(stream)))


def confspec_cascade_scratch_bytes(max_B: int, max_T: int, max_blocks_per_seq_target: int) -> int:
    return int(lib.confspec_cascade_scratch_bytes(max_B, max_T, max_blocks_per_seq_target))


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def confspec_cascade(draft_ctx, draft_w: Weights, draft_kv: KV, draft_ws, target_ctx, target_w: Weights, target_kv: KV,
                     target_ws, batch: Batch, requests: Requests, verdict_ids: Sequence[int], gamma: float, scratch,
                     out: CascadeOut, stream=None) -> int:
    """Returns the number of traces the large model's pass held."""
    nv = len(verdict_ids)
    ids = (C.c_int32 * max(nv, 1))(*[int(v) for v in verdict_ids])
    n_target = C.c_int32(0)
    _check(draft_ctx, lib.confspec_cascade(draft_ctx, C.byref(draft_w), C.byref(draft_kv), _ptr(draft_ws), _nbytes(draft_ws),
                                           target_ctx, C.byref(target_w), C.byref(target_kv), _ptr(target_ws),
                                           _nbytes(target_ws), C.byref(batch), C.byref(requests), ids, nv, float(gamma),
                                           _ptr(scratch), _nbytes(scratch), C.byref(out), C.byref(n_target),
                                           _stream_handle(stream)))
    return int(n_target.value)


def make_requests(req_start, h_req_start, parent=None, h_parent=None):
    """req_start: device int32 tensor [R+1]; h_req_start: the same values on the host; parent / h_parent: the
    candidate trees (device tensor [B] and host copy) or None for chains.  Returns (Requests, keepalive)."""
    import numpy as np
    hr = np.ascontiguousarray(h_req_start, dtype=np.int32)
    hp = None if h_parent is None else np.ascontiguousarray(h_parent, dtype=np.int32)
    hp_ptr = None if hp is None else hp.ctypes.data_as(C.POINTER(C.c_int32))
    return Requests(len(hr) - 1, _ptr(req_start), hr.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(parent), hp_ptr), (hr, hp)


PHASES = ("norm", "qkv", "attn", "attn_precise", "attn_merge", "o_proj", "gate_up", "down", "other")


def confspec_phase_timing(ctx, enable: bool) -> None:
    _check(ctx, lib.confspec_phase_timing(ctx, 1 if enable else 0))


def confspec_phase_times(ctx):
    """{phase name: (milliseconds, intervals)} of the most recent pass on the context (waits for it)."""
    ms = (C.c_float * len(PHASES))()
    n = (C.c_int32 * len(PHASES))()
    _check(ctx, lib.confspec_phase_times(ctx, ms, n))
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(PHASES)}


def confspec_tune(ctx, key: str, value: int) -> None:
    """ctx: a context, or None for the defaults of contexts created afterwards."""
    rc = lib.confspec_tune(ctx, key.encode(), int(value))
    if rc != OK:
        raise ConfSpecError(rc, f"confspec_tune({key!r}, {value})")


# --------------------------------------------------------------------------- #
# struct builders from torch tensors (pointer plumbing)
# --------------------------------------------------------------------------- #
def make_model_cfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_theta, rms_eps,
                   dtype: str) -> ModelCfg:
    return ModelCfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, float(rope_theta),
                    float(rms_eps), {"fp32": DTYPE_FP32, "bf16": DTYPE_BF16}[dtype])


def _ptr_array(tensors) -> "C.Array":
    arr = (C.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def make_weights(embed, lm_head, final_norm, attn_norm, wqkv, wo, mlp_norm, w_gate_up, w_down, packed=0):
    """Returns (Weights, keepalive): keepalive holds the host pointer arrays the struct points into."""
    arrays = [_ptr_array(x) for x in (attn_norm, wqkv, wo, mlp_norm, w_gate_up, w_down)]
    w = Weights(embed.data_ptr(), lm_head.data_ptr(), final_norm.data_ptr(),
                *[C.cast(a, C.POINTER(C.c_void_p)) for a in arrays], packed)
    return w, arrays


def make_kv(k_pages, v_pages, block_table, n_blocks: int, block_size: int, max_blocks_per_seq: int) -> KV:
    return KV(_ptr(k_pages), _ptr(v_pages), n_blocks, block_size, _ptr(block_table), max_blocks_per_seq)


def make_batch(suffix_ids, cu_suffix, prefix_lens, h_cu_suffix, h_prefix_lens):
    """h_cu_suffix / h_prefix_lens: int32 numpy arrays.  Returns (Batch, keepalive)."""
    import numpy as np
    hc = np.ascontiguousarray(h_cu_suffix, dtype=np.int32)
    hp = np.ascontiguousarray(h_prefix_lens, dtype=np.int32)
    B = len(hp)
    b = Batch(B, int(hc[-1]) if len(hc) else 0, _ptr(suffix_ids), _ptr(cu_suffix), _ptr(prefix_lens),
              hc.ctypes.data_as(C.POINTER(C.c_int32)), hp.ctypes.data_as(C.POINTER(C.c_int32)))
    return b, (hc, hp)
