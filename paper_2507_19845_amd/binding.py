"""ctypes binding of libgptstage.so (declared in include/gpt_stage.h).

Argument marshalling only: every function here has the name of the C entry
point it calls, takes torch tensors (used purely as device memory) or raw
integers, and forwards pointers.  No arithmetic of the stage runs in Python.
If the shared library has not been built this module raises at load time;
there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

import numpy as np
import torch

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgptstage.so")

GPTS_FP32, GPTS_BF16 = 0, 1
GPTS_GELU_TANH, GPTS_GELU_ERF = 0, 1
GPTS_OK, GPTS_EINVAL, GPTS_ESHAPE, GPTS_EHIP = 0, -1, -2, -3
N_TENSORS = 12

EXPORTS = (
    "gpt_stage_validate", "gpt_stage_param_count", "gpt_stage_param_bytes", "gpt_stage_grad_bytes",
    "gpt_stage_stash_bytes", "gpt_stage_workspace_bytes", "gpt_stage_param_offset",
    "gpt_stage_model_flops", "gpt_stage_strerror", "gpt_stage_prepared_bytes", "gpt_stage_prepare",
    "gpt_stage_fwd", "gpt_stage_bwd", "gpt_stage_fwd_only", "gpt_stage_bwd_only", "gpt_stage_fwd_bwd",
    "gpt_stage_grad_stash_bytes", "gpt_stage_bwd_data_only", "gpt_stage_wgrad_flush",
    "gpt_stage_op_layernorm_fwd", "gpt_stage_op_layernorm_bwd_scratch_bytes",
    "gpt_stage_op_layernorm_bwd", "gpt_stage_op_gemm", "gpt_stage_op_colsum_scratch_bytes",
    "gpt_stage_op_colsum", "gpt_stage_op_colsum_noalloc", "gpt_stage_op_attention_scratch_bytes", "gpt_stage_op_attention_fwd",
    "gpt_stage_op_attention_bwd",
    "gpt_stage_trace_create", "gpt_stage_trace_destroy", "gpt_stage_trace_reset",
    "gpt_stage_trace_collect", "gpt_stage_trace_op_name",
    "gpt_dpp_plan", "gpt_dpp_stash_slot_bytes", "gpt_dpp_grad_slot_bytes", "gpt_dpp_act_slot_bytes", "gpt_dpp_run",
    "gpt_dpp_allowance_from_free_memory", "gpt_dpp_simulate_ready", "gpt_dpp_run_ready",
    "gpt_fbd_coord_create", "gpt_fbd_coord_destroy", "gpt_fbd_coord_expected", "gpt_fbd_coord_register",
    "gpt_fbd_coord_align", "gpt_fbd_coord_ready", "gpt_fbd_coord_execute", "gpt_fbd_coord_simulate",
)


class gpt_stage_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("seq", C.c_int32),
                ("batch", C.c_int32), ("dtype", C.c_int32), ("gelu", C.c_int32),
                ("ln_eps", C.c_float), ("recompute", C.c_int32), ("fwd_fp16", C.c_int32)]


class gpt_stage_params(C.Structure):
    _fields_ = [("cfg", gpt_stage_cfg), ("weights", C.c_void_p), ("workspace", C.c_void_p),
                ("prepared", C.c_void_p), ("trace", C.c_void_p)]


class gpt_stage_trace_rec(C.Structure):
    _fields_ = [("op", C.c_int32), ("sub", C.c_int32), ("layer", C.c_int32), ("phase", C.c_int32),
                ("start_ms", C.c_float), ("dur_ms", C.c_float), ("flops", C.c_double),
                ("bytes", C.c_double)]


class gpt_dpp_task(C.Structure):
    _fields_ = [("phase", C.c_int32), ("microbatch", C.c_int32), ("chunk", C.c_int32)]


class gpt_dpp_job(C.Structure):
    _fields_ = [("n_chunks", C.c_int32), ("n_microbatches", C.c_int32), ("policy", C.c_int32),
                ("max_live_stash", C.c_int32), ("chunks", C.POINTER(gpt_stage_params)),
                ("x", C.POINTER(C.c_void_p)), ("dy", C.POINTER(C.c_void_p)),
                ("y", C.POINTER(C.c_void_p)), ("dx", C.POINTER(C.c_void_p)),
                ("dparams", C.POINTER(C.c_void_p)), ("stash_pool", C.c_void_p),
                ("stash_pool_bytes", C.c_size_t), ("act_pool", C.c_void_p),
                ("act_pool_bytes", C.c_size_t), ("grad_ready", C.POINTER(C.c_void_p)),
                ("grad_pool", C.c_void_p), ("grad_pool_bytes", C.c_size_t)]


class gpt_dpp_report(C.Structure):
    _fields_ = [("n_tasks", C.c_int32), ("peak_live_stash", C.c_int32), ("peak_live_act", C.c_int32),
                ("stash_slot_bytes", C.c_size_t), ("act_slot_bytes", C.c_size_t)]


GPT_DPP_DFC, GPT_DPP_BFC, GPT_DPP_BFC_BEST_EFFORT = 0, 1, 2
GPT_DPP_FWD, GPT_DPP_BWD = 0, 1
GPTS_ENOMEM = -4


class GptStageError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libgptstage error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once).  Fails loudly when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2507_19845_amd.build`")
    # a library built from other sources than the ones beside it would make every parity
    # statement meaningless: refuse it (the stamp is written by paper_2507_19845_amd.build)
    stamp = LIB_PATH + ".srchash"
    if os.path.exists(stamp) and os.path.isdir(os.path.join(_HERE, "csrc")):
        from . import build as _build
        if open(stamp).read().strip() != _build.source_hash():
            raise RuntimeError(f"{LIB_PATH} is older than its sources: rebuild with "
                               "`python -m paper_2507_19845_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz, f32 = C.c_void_p, C.c_int, C.c_size_t, C.c_float
    cfgp, parp = C.POINTER(gpt_stage_cfg), C.POINTER(gpt_stage_params)
    i32p = C.POINTER(C.c_int32)
    sig = {
        "gpt_stage_validate": (i32, [cfgp]),
        "gpt_stage_param_count": (sz, [cfgp]),
        "gpt_stage_param_bytes": (sz, [cfgp]),
        "gpt_stage_grad_bytes": (sz, [cfgp]),
        "gpt_stage_stash_bytes": (sz, [cfgp]),
        "gpt_stage_workspace_bytes": (sz, [cfgp, i32]),
        "gpt_stage_param_offset": (i32, [cfgp, i32, i32, C.POINTER(sz), C.POINTER(sz)]),
        "gpt_stage_model_flops": (C.c_double, [cfgp, i32]),
        "gpt_stage_strerror": (C.c_char_p, [i32]),
        "gpt_stage_prepared_bytes": (sz, [cfgp]),
        "gpt_stage_prepare": (i32, [parp, vp, vp]),
        "gpt_stage_fwd": (i32, [parp, vp, vp, vp, vp]),
        "gpt_stage_bwd": (i32, [parp, vp, vp, vp, vp, vp]),
        "gpt_stage_fwd_only": (i32, [parp, vp, vp, vp, vp, vp]),
        "gpt_stage_bwd_only": (i32, [parp, vp, vp, vp, vp, vp, vp]),
        "gpt_stage_fwd_bwd": (i32, [parp, vp, vp, vp, vp, vp, vp, vp]),
        "gpt_stage_grad_stash_bytes": (sz, [cfgp]),
        "gpt_stage_bwd_data_only": (i32, [parp, vp, vp, vp, vp, vp, vp, vp]),
        "gpt_stage_wgrad_flush": (i32, [parp, i32, C.POINTER(vp), C.POINTER(vp), vp, vp]),
        "gpt_stage_op_layernorm_fwd": (i32, [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp]),
        "gpt_stage_op_layernorm_bwd_scratch_bytes": (sz, [i32, i32]),
        "gpt_stage_op_layernorm_bwd": (i32, [i32, i32, i32, i32] + [vp] * 12),
        "gpt_stage_op_gemm": (i32, [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp]),
        "gpt_stage_op_colsum_scratch_bytes": (sz, [i32, i32]),
        "gpt_stage_op_colsum": (i32, [i32, i32, i32, vp, vp, vp, vp]),
        "gpt_stage_op_colsum_noalloc": (i32, [i32, i32, i32, vp, vp, vp]),
        "gpt_stage_op_attention_scratch_bytes": (sz, [i32, i32, i32, i32, i32, i32]),
        "gpt_stage_op_attention_fwd": (i32, [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]),
        "gpt_stage_op_attention_bwd": (i32, [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "gpt_stage_trace_create": (i32, [i32, C.POINTER(vp)]),
        "gpt_stage_trace_destroy": (i32, [vp]),
        "gpt_stage_trace_reset": (i32, [vp]),
        "gpt_stage_trace_collect": (i32, [vp, C.POINTER(gpt_stage_trace_rec), i32, C.POINTER(i32),
                                          C.POINTER(i32)]),
        "gpt_stage_trace_op_name": (C.c_char_p, [i32]),
        "gpt_dpp_plan": (i32, [i32, i32, i32, i32, C.POINTER(gpt_dpp_task), i32, C.POINTER(i32)]),
        "gpt_dpp_stash_slot_bytes": (sz, [parp, i32]),
        "gpt_dpp_grad_slot_bytes": (sz, [parp, i32]),
        "gpt_dpp_act_slot_bytes": (sz, [cfgp]),
        "gpt_dpp_run": (i32, [C.POINTER(gpt_dpp_job), vp, C.POINTER(gpt_dpp_report)]),
        "gpt_dpp_allowance_from_free_memory": (i32, [parp, i32, i32, sz, C.POINTER(sz), C.POINTER(sz)]),
        "gpt_dpp_simulate_ready": (i32, [i32, i32, i32, i32, i32p, i32p, i32, C.POINTER(gpt_dpp_task), i32, i32p, i32p]),
        "gpt_dpp_run_ready": (i32, [C.POINTER(gpt_dpp_job), C.POINTER(vp), C.POINTER(vp), C.c_double, vp,
                                    C.POINTER(gpt_dpp_task), i32, C.POINTER(gpt_dpp_report)]),
        "gpt_fbd_coord_create": (i32, [i32, i32, i32p, i32p, i32, i32p, C.POINTER(vp)]),
        "gpt_fbd_coord_destroy": (i32, [vp]),
        "gpt_fbd_coord_expected": (i32, [vp, i32, C.c_char_p]),
        "gpt_fbd_coord_register": (i32, [vp, i32, i32]),
        "gpt_fbd_coord_align": (i32, [vp]),
        "gpt_fbd_coord_ready": (i32, [vp, i32, i32p, i32]),
        "gpt_fbd_coord_execute": (i32, [vp, i32p, i32]),
        "gpt_fbd_coord_simulate": (i32, [vp, i32p, i32p, i32, i32p, i32, i32p, i32p]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != GPTS_OK:
        raise GptStageError(rc, lib().gpt_stage_strerror(rc).decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _event(ev: Optional[torch.cuda.Event]) -> Optional[int]:
    if ev is None:
        return None
    h = ev.cuda_event
    if not h:
        raise ValueError("torch.cuda.Event has no hipEvent yet: record it once before passing it")
    return h


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def make_cfg(s: synth.StageShape) -> gpt_stage_cfg:
    return gpt_stage_cfg(n_layers=s.n_layers, hidden=s.hidden, n_heads=s.n_heads, head_dim=s.head_dim,
                         ffn=s.ffn, seq=s.seq, batch=s.batch,
                         dtype=GPTS_BF16 if s.dtype == "bf16" else GPTS_FP32,
                         gelu=GPTS_GELU_ERF if s.gelu == "erf" else GPTS_GELU_TANH,
                         ln_eps=s.ln_eps, recompute=int(s.recompute),
                         fwd_fp16=1 if s.fwd_fp16 else 0)


# ---- host-side queries --------------------------------------------------------
def gpt_stage_validate(cfg: gpt_stage_cfg) -> int:
    return lib().gpt_stage_validate(C.byref(cfg))


def gpt_stage_param_count(cfg) -> int:
    return lib().gpt_stage_param_count(C.byref(cfg))


def gpt_stage_param_bytes(cfg) -> int:
    return lib().gpt_stage_param_bytes(C.byref(cfg))


def gpt_stage_grad_bytes(cfg) -> int:
    return lib().gpt_stage_grad_bytes(C.byref(cfg))


def gpt_stage_stash_bytes(cfg) -> int:
    return lib().gpt_stage_stash_bytes(C.byref(cfg))


def gpt_stage_workspace_bytes(cfg, phase: int) -> int:
    return lib().gpt_stage_workspace_bytes(C.byref(cfg), phase)


def gpt_stage_param_offset(cfg, layer: int, tensor_id: int):
    off, n = C.c_size_t(), C.c_size_t()
    _check(lib().gpt_stage_param_offset(C.byref(cfg), layer, tensor_id, C.byref(off), C.byref(n)))
    return off.value, n.value


def gpt_stage_model_flops(cfg, causal_aware: bool = True) -> float:
    return lib().gpt_stage_model_flops(C.byref(cfg), 1 if causal_aware else 0)


def gpt_stage_strerror(code: int) -> str:
    return lib().gpt_stage_strerror(code).decode()


# ---- the stage calls -----------------------------------------------------------
def make_params(cfg, weights, workspace, prepared=None, trace: Optional[int] = None) -> gpt_stage_params:
    """The C struct gpt_stage_params from tensors (pointers only: the caller keeps the
    tensors alive for as long as the struct is used)."""
    return gpt_stage_params(cfg=cfg, weights=_ptr(weights), workspace=_ptr(workspace),
                            prepared=_ptr(prepared), trace=trace)


def gpt_stage_prepared_bytes(cfg) -> int:
    return lib().gpt_stage_prepared_bytes(C.byref(cfg))


def gpt_stage_prepare(p: gpt_stage_params, prepared, stream=None) -> None:
    _check(lib().gpt_stage_prepare(C.byref(p), _ptr(prepared), _stream(stream)))


def gpt_stage_fwd(p: gpt_stage_params, x, act_stash, y, stream=None) -> None:
    _check(lib().gpt_stage_fwd(C.byref(p), _ptr(x), _ptr(act_stash), _ptr(y), _stream(stream)))


def gpt_stage_bwd(p: gpt_stage_params, act_stash, dy, dx, dparams, stream=None) -> None:
    _check(lib().gpt_stage_bwd(C.byref(p), _ptr(act_stash), _ptr(dy), _ptr(dx), _ptr(dparams),
                               _stream(stream)))


def gpt_stage_fwd_only(p: gpt_stage_params, x, act_stash, y, stream=None,
                       done_event: Optional[torch.cuda.Event] = None) -> None:
    ev = _event(done_event)
    _check(lib().gpt_stage_fwd_only(C.byref(p), _ptr(x), _ptr(act_stash), _ptr(y), _stream(stream), ev))


def gpt_stage_bwd_only(p: gpt_stage_params, act_stash, dy, dx, dparams, stream=None,
                       wait_event: Optional[torch.cuda.Event] = None) -> None:
    ev = _event(wait_event)
    _check(lib().gpt_stage_bwd_only(C.byref(p), _ptr(act_stash), _ptr(dy), _ptr(dx), _ptr(dparams),
                                    _stream(stream), ev))


def gpt_stage_grad_stash_bytes(cfg) -> int:
    return lib().gpt_stage_grad_stash_bytes(C.byref(cfg))


def gpt_stage_bwd_data_only(p: gpt_stage_params, act_stash, dy, dx, dparams, grad_stash, stream=None,
                            wait_event: Optional[torch.cuda.Event] = None) -> None:
    ev = _event(wait_event)
    _check(lib().gpt_stage_bwd_data_only(C.byref(p), _ptr(act_stash), _ptr(dy), _ptr(dx), _ptr(dparams),
                                         _ptr(grad_stash), _stream(stream), ev))


def gpt_stage_wgrad_flush(p: gpt_stage_params, act_stashes, grad_stashes, dparams, stream=None) -> None:
    n = len(act_stashes)
    assert len(grad_stashes) == n
    a, g = (C.c_void_p * n)(*[_ptr(t) for t in act_stashes]), (C.c_void_p * n)(*[_ptr(t) for t in grad_stashes])
    _check(lib().gpt_stage_wgrad_flush(C.byref(p), n, a, g, _ptr(dparams), _stream(stream)))


def gpt_stage_fwd_bwd(p: gpt_stage_params, x, dy, act_stash, y, dx, dparams, stream=None) -> None:
    _check(lib().gpt_stage_fwd_bwd(C.byref(p), _ptr(x), _ptr(dy), _ptr(act_stash), _ptr(y), _ptr(dx),
                                   _ptr(dparams), _stream(stream)))


# ---- operator tracer --------------------------------------------------------------
def gpt_stage_trace_create(capacity: int) -> int:
    h = C.c_void_p()
    _check(lib().gpt_stage_trace_create(capacity, C.byref(h)))
    return h.value


def gpt_stage_trace_destroy(trace: int) -> None:
    _check(lib().gpt_stage_trace_destroy(trace))


def gpt_stage_trace_reset(trace: int) -> None:
    _check(lib().gpt_stage_trace_reset(trace))


def gpt_stage_trace_collect(trace: int, max_records: int):
    """Returns (list of record dicts in launch order, number of dropped records)."""
    buf = (gpt_stage_trace_rec * max_records)()
    n, dropped = C.c_int(), C.c_int()
    _check(lib().gpt_stage_trace_collect(trace, buf, max_records, C.byref(n), C.byref(dropped)))
    recs = [dict(op=gpt_stage_trace_op_name(r.op), sub=r.sub, layer=r.layer, phase=r.phase,
                 start_ms=r.start_ms, dur_ms=r.dur_ms, flops=r.flops, bytes=r.bytes)
            for r in buf[:n.value]]
    return recs, dropped.value


def gpt_stage_trace_op_name(op: int) -> str:
    return lib().gpt_stage_trace_op_name(op).decode()


# ---- single operations ----------------------------------------------------------
def gpt_stage_op_layernorm_fwd(dtype, T, H, eps, x, gamma, beta, out, mean, rstd, stream=None, x_f32=False):
    _check(lib().gpt_stage_op_layernorm_fwd(dtype, int(x_f32), T, H, eps, _ptr(x), _ptr(gamma), _ptr(beta),
                                            _ptr(out), _ptr(mean), _ptr(rstd), _stream(stream)))


def gpt_stage_op_layernorm_bwd_scratch_bytes(T, H) -> int:
    return lib().gpt_stage_op_layernorm_bwd_scratch_bytes(T, H)


def gpt_stage_op_layernorm_bwd(dtype, T, H, dout, x, mean, rstd, gamma, dres, dx, dgamma, dbeta,
                               partial, stream=None, x_f32=False, dxsum=None):
    _check(lib().gpt_stage_op_layernorm_bwd(dtype, int(x_f32), T, H, _ptr(dout), _ptr(x), _ptr(mean), _ptr(rstd),
                                            _ptr(gamma), _ptr(dres), _ptr(dx), _ptr(dgamma),
                                            _ptr(dbeta), _ptr(dxsum), _ptr(partial), _stream(stream)))


def gpt_stage_op_gemm(dtype, form, M, N, K, A, B, Cout, bias=None, residual=None, C2=None,
                      dgelu_u=None, gelu_kind=GPTS_GELU_TANH, stream=None, f32_flags=0):
    _check(lib().gpt_stage_op_gemm(dtype, form, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(bias),
                                   _ptr(residual), _ptr(C2), _ptr(dgelu_u), gelu_kind, f32_flags,
                                   _stream(stream)))


def gpt_stage_op_colsum_scratch_bytes(M, N) -> int:
    return lib().gpt_stage_op_colsum_scratch_bytes(M, N)


def gpt_stage_op_colsum(dtype, M, N, A, colsum, partial, stream=None):
    _check(lib().gpt_stage_op_colsum(dtype, M, N, _ptr(A), _ptr(colsum), _ptr(partial), _stream(stream)))


def gpt_stage_op_colsum_noalloc(dtype, M, N, A, colsum, stream=None):
    _check(lib().gpt_stage_op_colsum_noalloc(dtype, M, N, _ptr(A), _ptr(colsum), _stream(stream)))


def gpt_stage_op_attention_scratch_bytes(dtype, B, S, n_heads, head_dim, phase: int) -> int:
    return lib().gpt_stage_op_attention_scratch_bytes(dtype, B, S, n_heads, head_dim, phase)


def gpt_stage_op_attention_fwd(dtype, B, S, n_heads, head_dim, qkv, out, lse, scratch, stream=None):
    _check(lib().gpt_stage_op_attention_fwd(dtype, B, S, n_heads, head_dim, _ptr(qkv), _ptr(out),
                                            _ptr(lse), _ptr(scratch), _stream(stream)))


def gpt_stage_op_attention_bwd(dtype, B, S, n_heads, head_dim, qkv, out, lse, dout, dqkv, scratch,
                               stream=None):
    _check(lib().gpt_stage_op_attention_bwd(dtype, B, S, n_heads, head_dim, _ptr(qkv), _ptr(out),
                                            _ptr(lse), _ptr(dout), _ptr(dqkv), _ptr(scratch),
                                            _stream(stream)))


# ---- traversal of the (micro-batch, chunk) task matrix ---------------------------------
def gpt_dpp_plan(policy: int, n_chunks: int, n_microbatches: int, max_live_stash: int = 0):
    """-> ([(phase, microbatch, chunk), ...], peak_live_stash)"""
    cap = 2 * max(n_chunks, 0) * max(n_microbatches, 0)
    arr = (gpt_dpp_task * max(cap, 1))()
    peak = C.c_int(0)
    n = lib().gpt_dpp_plan(policy, n_chunks, n_microbatches, max_live_stash, arr, cap, C.byref(peak))
    if n < 0:
        _check(n)
    return [(arr[k].phase, arr[k].microbatch, arr[k].chunk) for k in range(n)], peak.value


def _params_array(chunks):
    arr = (gpt_stage_params * len(chunks))()
    for k, c in enumerate(chunks):
        arr[k] = c
    return arr


def gpt_dpp_stash_slot_bytes(chunks) -> int:
    return lib().gpt_dpp_stash_slot_bytes(_params_array(chunks), len(chunks))


def gpt_dpp_grad_slot_bytes(chunks) -> int:
    return lib().gpt_dpp_grad_slot_bytes(_params_array(chunks), len(chunks))


def gpt_dpp_act_slot_bytes(cfg) -> int:
    return lib().gpt_dpp_act_slot_bytes(C.byref(cfg))


def gpt_dpp_allowance_from_free_memory(chunks, n_microbatches: int, reserve_bytes: int = 0):
    """-> (allowance, stash_pool_bytes, act_pool_bytes)"""
    sp, ap = C.c_size_t(), C.c_size_t()
    n = lib().gpt_dpp_allowance_from_free_memory(_params_array(chunks), len(chunks), n_microbatches,
                                                 reserve_bytes, C.byref(sp), C.byref(ap))
    if n < 0:
        _check(n)
    return n, sp.value, ap.value


def gpt_dpp_simulate_ready(policy: int, n_chunks: int, n_microbatches: int, max_live_stash: int = 0,
                           x_at=None, dy_at=None, dynamic: bool = True):
    """-> ([(phase, microbatch, chunk), ...] in order of issue, n_steps, idle_steps)"""
    cap = 2 * max(n_chunks, 0) * max(n_microbatches, 0)
    arr = (gpt_dpp_task * max(cap, 1))()
    steps, idle = C.c_int32(0), C.c_int32(0)
    xa = _i32(list(x_at)) if x_at is not None else None
    da = _i32(list(dy_at)) if dy_at is not None else None
    n = lib().gpt_dpp_simulate_ready(policy, n_chunks, n_microbatches, max_live_stash, xa, da,
                                     1 if dynamic else 0, arr, cap, C.byref(steps), C.byref(idle))
    if n < 0:
        _check(n)
    return [(arr[k].phase, arr[k].microbatch, arr[k].chunk) for k in range(n)], steps.value, idle.value


def _dpp_job(policy, chunks, xs, dys, ys, dxs, dparams, stash_pool, act_pool, max_live_stash, grad_ready,
             grad_pool=None):
    def ptrs(ts):
        a = (C.c_void_p * len(ts))()
        for k, t in enumerate(ts):
            a[k] = _ptr(t)
        return a
    keep = [_params_array(chunks), ptrs(xs), ptrs(dys), ptrs(ys), ptrs(dxs), ptrs(dparams)]
    ev = None
    if grad_ready is not None:
        ev = (C.c_void_p * len(grad_ready))()
        for k, e in enumerate(grad_ready):
            ev[k] = _event(e)
    job = gpt_dpp_job(n_chunks=len(chunks), n_microbatches=len(xs), policy=policy,
                      max_live_stash=max_live_stash, chunks=keep[0], x=keep[1], dy=keep[2],
                      y=keep[3], dx=keep[4], dparams=keep[5],
                      stash_pool=_ptr(stash_pool), stash_pool_bytes=stash_pool.numel() if stash_pool is not None else 0,
                      act_pool=_ptr(act_pool), act_pool_bytes=act_pool.numel() if act_pool is not None else 0,
                      grad_ready=ev, grad_pool=_ptr(grad_pool),
                      grad_pool_bytes=grad_pool.numel() if grad_pool is not None else 0)
    return job, keep + [ev]


def gpt_dpp_run_ready(policy: int, chunks, xs, dys, ys, dxs, dparams, stash_pool, act_pool,
                      x_ready=None, dy_ready=None, max_live_stash: int = 0, timeout_seconds: float = 30.0,
                      grad_ready=None, stream=None):
    """x_ready / dy_ready: None or one torch.cuda.Event (or None) per micro-batch.
    -> (gpt_dpp_report, [(phase, microbatch, chunk), ...] in order of issue)"""
    job, keep = _dpp_job(policy, chunks, xs, dys, ys, dxs, dparams, stash_pool, act_pool, max_live_stash, grad_ready)

    def events(evs):
        if evs is None:
            return None
        a = (C.c_void_p * len(evs))()
        for k, e in enumerate(evs):
            a[k] = _event(e) if e is not None else None
        return a
    xe, de = events(x_ready), events(dy_ready)
    cap = 2 * len(chunks) * len(xs)
    order = (gpt_dpp_task * cap)()
    rep = gpt_dpp_report()
    _check(lib().gpt_dpp_run_ready(C.byref(job), xe, de, timeout_seconds, _stream(stream), order, cap, C.byref(rep)))
    return rep, [(order[k].phase, order[k].microbatch, order[k].chunk) for k in range(rep.n_tasks)]


def gpt_dpp_run(policy: int, chunks, xs, dys, ys, dxs, dparams, stash_pool, act_pool,
                max_live_stash: int = 0, grad_ready=None, stream=None, grad_pool=None) -> gpt_dpp_report:
    """chunks: list of gpt_stage_params; xs, dys, ys, dxs: one tensor per micro-batch;
    dparams: one fp32 tensor per chunk; stash_pool / act_pool: uint8 tensors (act_pool may be
    None for a single chunk); grad_ready: None or one torch.cuda.Event per chunk; grad_pool:
    None, or a uint8 tensor of gradient-stash slots (one weight phase per chunk and window)."""
    job, keep = _dpp_job(policy, chunks, xs, dys, ys, dxs, dparams, stash_pool, act_pool, max_live_stash,
                         grad_ready, grad_pool)
    rep = gpt_dpp_report()
    _check(lib().gpt_dpp_run(C.byref(job), _stream(stream), C.byref(rep)))
    return rep


# ---- communication coordinator, simulated on the host ---------------------------------
def _i32(values):
    return (C.c_int32 * max(len(values), 1))(*values)


def _ragged(lists):
    start, flat = [0], []
    for l in lists:
        flat += list(l)
        start.append(len(flat))
    return _i32(start), _i32(flat)


def gpt_fbd_coord_create(n_ranks: int, groups, control_of_rank) -> int:
    """groups: list of member lists; control_of_rank: control thread of each virtual rank.
    Returns the coordinator handle."""
    gs, gm = _ragged(groups)
    h = C.c_void_p()
    _check(lib().gpt_fbd_coord_create(n_ranks, len(groups), gs, gm, max(control_of_rank) + 1 if control_of_rank else 0,
                                      _i32(list(control_of_rank)), C.byref(h)))
    return h.value


def gpt_fbd_coord_destroy(coord) -> None:
    _check(lib().gpt_fbd_coord_destroy(coord))


def gpt_fbd_coord_expected(coord, group: int, n_ranks: int) -> str:
    buf = C.create_string_buffer(n_ranks + 1)
    _check(lib().gpt_fbd_coord_expected(coord, group, buf))
    return buf.value.decode()


def gpt_fbd_coord_register(coord, rank: int, group: int) -> None:
    _check(lib().gpt_fbd_coord_register(coord, rank, group))


def gpt_fbd_coord_align(coord) -> None:
    _check(lib().gpt_fbd_coord_align(coord))


def gpt_fbd_coord_ready(coord, control: int, n_groups: int):
    out = (C.c_int32 * max(n_groups, 1))()
    n = lib().gpt_fbd_coord_ready(coord, control, out, n_groups)
    if n < 0:
        _check(n)
    return list(out[:n])


def gpt_fbd_coord_execute(coord, n_groups: int):
    out = (C.c_int32 * max(n_groups, 1))()
    n = lib().gpt_fbd_coord_execute(coord, out, n_groups)
    if n < 0:
        _check(n)
    return list(out[:n])


def gpt_fbd_coord_simulate(coord, programs, verify: bool):
    """-> (log, deadlocked)"""
    ps, pf = _ragged(programs)
    cap = max(sum(len(p) for p in programs), 1)
    log = (C.c_int32 * cap)()
    n, dead = C.c_int32(0), C.c_int32(0)
    _check(lib().gpt_fbd_coord_simulate(coord, ps, pf, 1 if verify else 0, log, cap, C.byref(n), C.byref(dead)))
    return list(log[:n.value]), bool(dead.value)


# ---- device-memory plumbing (torch tensors as buffers; no arithmetic) --------------
def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Upload an fp32 numpy array whose values are already representable in
    `dtype` ("fp32" or "bf16") as a tensor of that storage type."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = synth.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Download a tensor as float64 numpy (exact widening)."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


class StageBuffers:
    """Owns the device buffers one stage needs and moves parameters in and
    gradients out.  Pure allocation and copying."""

    def __init__(self, shape: synth.StageShape, n_stash: int = 1, device="cuda"):
        self.shape = shape
        self.cfg = make_cfg(shape)
        rc = gpt_stage_validate(self.cfg)
        if rc != GPTS_OK:
            raise GptStageError(rc, gpt_stage_strerror(rc))
        self.device = device
        self.tdtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.n_param = gpt_stage_param_count(self.cfg)
        self.weights = torch.zeros(self.n_param, dtype=self.tdtype, device=device)
        self.dparams = torch.zeros(self.n_param, dtype=torch.float32, device=device)
        # the slots are slices of one allocation, equally spaced: what the weight phase
        # (gpt_stage_wgrad_flush) needs to contract over all micro-batches in one product
        sb = gpt_stage_stash_bytes(self.cfg)
        self._stash_all = torch.empty(sb * n_stash, dtype=torch.uint8, device=device)
        self.stash = [self._stash_all[i * sb:(i + 1) * sb] for i in range(n_stash)]
        self.grad_stash: List[torch.Tensor] = []        # filled by alloc_grad_stash()
        wb = max(gpt_stage_workspace_bytes(self.cfg, 0), gpt_stage_workspace_bytes(self.cfg, 1), 256)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=device)
        self.prepared: Optional[torch.Tensor] = None    # passed as params.prepared when set
        self._prepared_buf: Optional[torch.Tensor] = None
        self.trace: Optional[int] = None                # tracer handle passed as params.trace

    def alloc_grad_stash(self, n: int) -> None:
        """n gradient-stash slots (slices of one allocation) for the split backward phase."""
        if len(self.grad_stash) >= n:
            return
        gb = gpt_stage_grad_stash_bytes(self.cfg)
        self._grad_all = torch.empty(gb * n, dtype=torch.uint8, device=self.device)
        self.grad_stash = [self._grad_all[i * gb:(i + 1) * gb] for i in range(n)]

    def params(self) -> gpt_stage_params:
        """gpt_stage_params for the stage calls: this object's weights and workspace, the
        prepared weights if prepare() was called, and the tracer in self.trace (if any)."""
        return make_params(self.cfg, self.weights, self.workspace, self.prepared, self.trace)

    def prepare(self, stream=None) -> None:
        """(Re)build the prepared-weights buffer from the current weights; it is passed
        with every later params() (bf16 stages only)."""
        nbytes = gpt_stage_prepared_bytes(self.cfg)
        if nbytes == 0:
            return
        if self._prepared_buf is None:
            self._prepared_buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        gpt_stage_prepare(make_params(self.cfg, self.weights, None), self._prepared_buf, stream)
        self.prepared = self._prepared_buf

    def unprepare(self) -> None:
        self.prepared = None

    def act(self) -> torch.Tensor:
        s = self.shape
        return torch.empty((s.batch, s.seq, s.hidden), dtype=self.tdtype, device=self.device)

    def load_params(self, params: List[Dict[str, np.ndarray]]) -> None:
        for l, p in enumerate(params):
            for tid, name in enumerate(synth.TENSOR_NAMES):
                off, n = gpt_stage_param_offset(self.cfg, l, tid)
                assert p[name].size == n, (name, p[name].shape, n)
                self.weights[off:off + n].copy_(to_device(p[name].reshape(-1), self.shape.dtype, self.device))
        if self.shape.fwd_fp16:
            self.prepare()   # the fp16 forward products read the weights through their images

    def read_grads(self) -> List[Dict[str, np.ndarray]]:
        shapes = synth.param_shapes(self.shape)
        flat = self.dparams.cpu().numpy()
        out = []
        for l in range(self.shape.n_layers):
            d = {}
            for tid, name in enumerate(synth.TENSOR_NAMES):
                off, n = gpt_stage_param_offset(self.cfg, l, tid)
                d[name] = flat[off:off + n].reshape(shapes[name]).astype(np.float64)
            out.append(d)
        return out
