"""Which roundings decide the error of the tensor-parallel-share workload (CPU only).

The workload has hidden 12288 and N(0, 0.02) weights, so its attention logits have a
standard deviation of ~5 and the softmax amplifies the rounding of whatever feeds them --
in the second layer that is every forward activation of the first.  The emulation
(tests/rounding_emulation.py) re-runs the oracle's arithmetic with the stage's rounding
points and shows, at a reduced sequence length:
  * bf16 forward activations put the gradients outside the 2e-2 bar;
  * lifting only the logit path (LayerNorm-1 output as q/k read it, q, k) -- even to exact
    arithmetic -- removes about half of the error, not enough for a margin at full length;
  * fp16 forward activations (cfg.fwd_fp16), with every backward rounding left at bf16,
    bring every tensor well inside the bar.
The full-length figures are in the design notes; the GPU test of the workload asserts the
bar itself.
"""
import math

import numpy as np

from oracle import gpt_stage_oracle as orc

import rounding_emulation as emu


def test_emulator_without_rounding_is_the_oracle():
    s, x, dy, params = emu.tp_share_inputs(64)
    s = s.with_(hidden=256, ffn=512)   # the emulator's arithmetic, not the workload: keep it small
    from paper_2507_19845_amd import synth
    params = [{k: v.astype(np.float64) for k, v in p.items()} for p in synth.make_params(s, 0)]
    x, dy = synth.make_x(s, 0).astype(np.float64), synth.make_dy(s, 0).astype(np.float64)
    ref = orc.stage_fwd_bwd(x, dy, params, s.n_heads, s.head_dim, s.ln_eps, s.gelu)
    got = emu.emulate(s, x, dy, params, {r: "exact" for r in emu.ROLES})
    assert max(emu.max_norm_errors(got, ref).values()) < 1e-12


def test_tp_share_workload_needs_fp16_forward_activations():
    s, x, dy, params = emu.tp_share_inputs(128)
    ref = orc.stage_fwd_bwd(x, dy, params, s.n_heads, s.head_dim, s.ln_eps, s.gelu)
    # the logits are large: that is what amplifies the rounding
    P, d = s.attn_width, s.head_dim
    a, _, _ = orc.layernorm_fwd(x, params[0]["ln1_g"], params[0]["ln1_b"], s.ln_eps)
    qkv = a @ params[0]["w_qkv"].T
    logits = qkv[0, :, :d] @ qkv[0, :, P:P + d].T / math.sqrt(d)
    assert 4.0 < logits.std() < 6.0
    worst = {}
    for name in ("bf16 everywhere (plain bf16 stage)", "exact logit path (a for q/k, q, k)",
                 "fp16 forward activations (cfg.fwd_fp16)"):
        e = emu.max_norm_errors(emu.emulate(s, x, dy, params, emu.CASES[name]), ref)
        worst[name] = max(e.values())
        print(f"{name}: {worst[name]:.3e}")
    plain, logit, fwd16 = worst.values()
    assert plain > 2e-2                      # a plain bf16 stage misses the bar
    assert logit > 0.35 * plain              # the logit path alone leaves too much
    assert fwd16 < 1.3e-2 and fwd16 < 0.45 * plain
