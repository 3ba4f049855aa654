"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, validates shapes, and its layout / FLOP
queries return the documented values."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2507_19845_amd import binding as B
from paper_2507_19845_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gpt_stage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gpt_(?:stage|dpp|fbd)_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 20
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in gpt_stage.h but not exported"
    assert sorted(B.EXPORTS) == names, "binding and header disagree on the entry points"


def test_binding_has_a_function_per_entry_point():
    for n in _declared():
        assert callable(getattr(B, n)), n


@pytest.mark.parametrize("shape", synth.WORKLOADS, ids=lambda s: s.name)
def test_workloads_validate_and_layout(shape):
    cfg = B.make_cfg(shape)
    assert B.gpt_stage_validate(cfg) == B.GPTS_OK
    n = B.gpt_stage_param_count(cfg)
    assert n == synth.params_per_layer(shape) * shape.n_layers
    assert B.gpt_stage_param_bytes(cfg) == n * (2 if shape.dtype == "bf16" else 4)
    assert B.gpt_stage_grad_bytes(cfg) == n * 4
    shapes = synth.param_shapes(shape)
    expect = 0
    for l in range(shape.n_layers):
        for tid, name in enumerate(synth.TENSOR_NAMES):
            off, cnt = B.gpt_stage_param_offset(cfg, l, tid)
            assert off == expect and cnt == int(np.prod(shapes[name])) and off % 8 == 0
            expect += cnt
    assert B.gpt_stage_stash_bytes(cfg) > 0
    assert B.gpt_stage_workspace_bytes(cfg, 1) > 0


def test_model_flops_match_the_formula():
    # per layer forward: 2 T (3PH + PH + 2HF) + 4 B a d S(S+1)/2, x3 for fwd+bwd
    want_tf = {0: 0.157e-3, 1: 1.340, 2: 7.989, 3: 171.5 / 8, 4: 5.644}   # causal-aware, per micro-batch
    want_dense = {0: 0.164e-3, 1: 1.443, 2: 8.246, 3: 184.7 / 8, 4: 5.721}
    for i, s in enumerate(synth.WORKLOADS):
        cfg = B.make_cfg(s)
        T, P, H, F = s.tokens, s.attn_width, s.hidden, s.ffn
        lin = 2 * T * (4 * P * H + 2 * H * F)
        att = 4 * s.batch * s.n_heads * s.head_dim * s.seq * (s.seq + 1) // 2
        assert B.gpt_stage_model_flops(cfg, True) == pytest.approx(3 * s.n_layers * (lin + att), rel=1e-12)
        assert B.gpt_stage_model_flops(cfg, True) / 1e12 == pytest.approx(want_tf[i], rel=5e-3)
        assert B.gpt_stage_model_flops(cfg, False) / 1e12 == pytest.approx(want_dense[i], rel=5e-3)


@pytest.mark.parametrize("field,value,code", [
    ("head_dim", 48, B.GPTS_ESHAPE), ("hidden", 100, B.GPTS_ESHAPE), ("hidden", 32768, B.GPTS_ESHAPE),
    ("n_layers", 0, B.GPTS_ESHAPE), ("dtype", 7, B.GPTS_EINVAL), ("gelu", 2, B.GPTS_EINVAL),
    ("seq", 0, B.GPTS_ESHAPE), ("ffn", 12, B.GPTS_ESHAPE),
])
def test_validate_rejects(field, value, code):
    cfg = B.make_cfg(synth.WORKLOADS[0])
    setattr(cfg, field, value)
    assert B.gpt_stage_validate(cfg) == code
    assert B.gpt_stage_strerror(code) not in ("ok", "")
    assert B.gpt_stage_param_count(cfg) == 0 and B.gpt_stage_stash_bytes(cfg) == 0


def test_strerror_depends_on_the_code():
    cfg = B.make_cfg(synth.WORKLOADS[0])
    cfg.head_dim = 48
    assert B.gpt_stage_validate(cfg) == B.GPTS_ESHAPE
    assert "head_dim" in B.gpt_stage_strerror(B.GPTS_ESHAPE)       # the last failure's own text
    assert "head_dim" not in B.gpt_stage_strerror(B.GPTS_EINVAL)   # another status: its generic meaning
    assert B.gpt_stage_strerror(B.GPTS_OK) == "ok"
    assert B.gpt_stage_strerror(-99) == "unknown status"
    texts = {B.gpt_stage_strerror(c) for c in (B.GPTS_EINVAL, B.GPTS_EHIP, B.GPTS_ENOMEM)}
    assert len(texts) == 3


def test_fwd_fp16_validation():
    ok = synth.WORKLOADS[4]
    assert ok.fwd_fp16 and B.gpt_stage_validate(B.make_cfg(ok)) == B.GPTS_OK
    assert B.gpt_stage_validate(B.make_cfg(ok.with_(ffn=6144 + 64))) == B.GPTS_ESHAPE      # not a multiple of 128
    assert B.gpt_stage_validate(B.make_cfg(synth.WORKLOADS[0].with_(fwd_fp16=True))) == B.GPTS_EINVAL  # fp32 stage
    assert B.gpt_stage_validate(B.make_cfg(ok.with_(head_dim=32, n_heads=48))) == B.GPTS_OK
    # same stash size as the recomputing layout: A, A2, G are not stashed, QKV / C / U are 16-bit either way
    plain = ok.with_(fwd_fp16=False)
    assert B.gpt_stage_stash_bytes(B.make_cfg(ok)) == B.gpt_stage_stash_bytes(B.make_cfg(plain.with_(recompute=True)))
    assert B.gpt_stage_stash_bytes(B.make_cfg(ok)) < B.gpt_stage_stash_bytes(B.make_cfg(plain))
    # the stage calls refuse to run without prepared weights
    cfg = B.make_cfg(ok)
    p = B.gpt_stage_params(cfg=cfg, weights=0x1000, workspace=0x2000)
    assert B.lib().gpt_stage_fwd(ctypes.byref(p), 0x3000, 0x4000, 0x5000, None) == B.GPTS_EINVAL
    assert "prepared" in B.gpt_stage_strerror(B.GPTS_EINVAL)


def test_recompute_levels_validate_and_shrink_the_stash():
    s = synth.WORKLOADS[3]
    sizes = [B.gpt_stage_stash_bytes(B.make_cfg(s.with_(recompute=r))) for r in (0, 1, 2)]
    assert sizes[0] > sizes[1] > sizes[2] == s.n_layers * s.tokens * s.hidden * 4
    assert B.gpt_stage_validate(B.make_cfg(s.with_(recompute=3))) == B.GPTS_EINVAL
    # level 2 moves the layer block into the workspaces
    w0 = [B.gpt_stage_workspace_bytes(B.make_cfg(s.with_(recompute=r)), 0) for r in (0, 2)]
    assert w0[1] - w0[0] >= sizes[0] // s.n_layers - s.tokens * s.hidden * 4 - 4096


def test_split_backward_is_refused_where_it_cannot_work():
    """Keep-only-x recomputation leaves no activations for a later weight phase: both halves of
    the split backward return GPTS_EINVAL before anything is launched (fake, aligned pointers)."""
    cfg = B.make_cfg(synth.WORKLOADS[1].with_(recompute=2))
    p = B.gpt_stage_params(cfg=cfg, weights=0x10000, workspace=0x20000)
    L = B.lib()
    assert L.gpt_stage_bwd_data_only(ctypes.byref(p), 0x30000, 0x40000, 0x50000, 0x60000, 0x70000, None, None) == B.GPTS_EINVAL
    assert "recompute" in B.gpt_stage_strerror(B.GPTS_EINVAL)
    arr = (ctypes.c_void_p * 1)(0x30000)
    assert L.gpt_stage_wgrad_flush(ctypes.byref(p), 1, arr, arr, 0x60000, None) == B.GPTS_EINVAL
    assert B.gpt_stage_grad_stash_bytes(cfg) > 0
    ok = B.make_cfg(synth.WORKLOADS[3])
    T, H, P, F, Ln = 4096, 4096, 4096, 16384, 4
    assert B.gpt_stage_grad_stash_bytes(ok) == Ln * (2 * T * H + T * F + T * 3 * P) * 2
    q = B.gpt_stage_params(cfg=ok, weights=0x10000, workspace=0x20000)
    assert L.gpt_stage_wgrad_flush(ctypes.byref(q), 0, arr, arr, 0x60000, None) == B.GPTS_EINVAL
    assert L.gpt_stage_bwd_data_only(ctypes.byref(q), 0x30000, 0x40000, 0x50000, 0x60000, None, None, None) == B.GPTS_EINVAL


def test_bf16_needs_tile_multiples():
    s = synth.WORKLOADS[1].with_(seq=1000, batch=1)
    assert B.gpt_stage_validate(B.make_cfg(s)) == B.GPTS_ESHAPE
    assert B.gpt_stage_validate(B.make_cfg(s.with_(dtype="fp32"))) == B.GPTS_OK


def test_calls_reject_null_pointers_without_touching_the_gpu():
    cfg = B.make_cfg(synth.WORKLOADS[0])
    p = B.gpt_stage_params(cfg=cfg, weights=None, workspace=None)
    L = B.lib()
    assert L.gpt_stage_fwd(ctypes.byref(p), None, None, None, None) == B.GPTS_EINVAL
    assert L.gpt_stage_bwd(ctypes.byref(p), None, None, None, None, None) == B.GPTS_EINVAL
    assert L.gpt_stage_fwd(None, None, None, None, None) == B.GPTS_EINVAL
    p.weights = 0x1008   # misaligned
    assert L.gpt_stage_fwd(ctypes.byref(p), 0x1000, 0x2000, 0x3000, None) == B.GPTS_EINVAL


def test_bf16_rounding_helper_is_round_to_nearest_even():
    import torch
    a = synth.make_aux(0, 1, (4096,), 3.0)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e38]   # two exact ties, sign, near-overflow
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(synth.round_to_bf16(a), want)
    assert np.array_equal(synth.bf16_bits_to_f32(synth.bf16_bits(want)), want)
