"""CPU emulation of where a bf16 stage rounds, built on the fp64 oracle's own functions.

The stage stores activations and activation gradients in 16 bits between kernels.  This
module re-runs the oracle's forward and backward arithmetic (same formulas, fp64) but
rounds each stored tensor at the point where the stage stores it, with a rounding mode
per tensor ROLE, so that one can ask which roundings an output's error comes from:

    bf16   8 significand bits (what a bf16 stage stores)
    fp16   11 significand bits
    split  hi + lo pair of bf16 values (16 significand bits)
    exact  no rounding

Roles (all default to bf16):
  forward    a_qk, a_v : LayerNorm-1 output as the Q/K resp. V columns of the qkv product read it
             q_s, k_s  : q, k as the attention logits read them (forward and backward recompute)
             v         : v as the forward P V product reads it;   p : probabilities fed to P V
             c         : attention output as the out-projection reads it
             c_delta   : attention output as delta = rowsum(dO * O) reads it
             a2, u, g  : LayerNorm-2 output, fc1 pre-activation (feeds gelu and gelu'), gelu output
             yout      : the stage output
  backward   a_w, a2_w, c_w : the copies the weight-gradient products read
             q_g, k_g, v_g  : q, k, v as dK = dS^T Q, dQ = dS K, dP = dO V^T read them
             pb, dS, dQ, dK, dV, dU, dA2, dX1, dC, dA, dX : gradient tensors as stored
The residual stream (x, x1, y between layers) is fp32 in the stage and exact here.

Run as a script to print the table for a sequence length (default 512):
    python tests/rounding_emulation.py [seq]
"""
from __future__ import annotations

import math
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))   # run as a script too

from oracle import gpt_stage_oracle as orc
from paper_2507_19845_amd import synth

ROLES = ("a_qk", "a_v", "a_w", "q_s", "k_s", "q_g", "k_g", "v", "v_g", "p", "c", "c_delta", "c_w",
         "a2", "a2_w", "u", "g", "yout", "dU", "dA2", "dX1", "dC", "pb", "dS", "dQ", "dK", "dV", "dA", "dX")


def _bf16(a):
    return synth.round_to_bf16(np.asarray(a, np.float32)).astype(np.float64)


def _fp16(a):
    return np.asarray(a, np.float32).astype(np.float16).astype(np.float64)


def _split(a):
    a32 = np.asarray(a, np.float32)
    hi = synth.round_to_bf16(a32)
    return hi.astype(np.float64) + synth.round_to_bf16(a32 - hi).astype(np.float64)


MODES = {"bf16": _bf16, "fp16": _fp16, "split": _split, "exact": lambda a: a}

# the forward activations a stage with cfg.fwd_fp16 keeps in fp16
FWD_FP16 = dict(a_qk="fp16", a_v="fp16", q_s="fp16", k_s="fp16", v="fp16", p="fp16", c="fp16",
                c_delta="fp16", a2="fp16", u="fp16", g="fp16")


def emulate(shape, x, dy, params, roles=None):
    """Forward + backward of the stage with per-role rounding.  Returns (y, dx, grads)."""
    m = {r: MODES["bf16"] for r in ROLES}
    for k, v in (roles or {}).items():
        assert k in m, k
        m[k] = MODES[v]
    P, d, L = shape.attn_width, shape.head_dim, len(params)
    B, S, _ = x.shape
    mask = np.tril(np.ones((S, S), bool))
    scale = 1.0 / math.sqrt(d)
    saved, h = [], np.asarray(x, np.float64)
    for l, p in enumerate(params):
        a, xh1, r1 = orc.layernorm_fwd(h, p["ln1_g"], p["ln1_b"], shape.ln_eps)
        aqk = m["a_qk"](a)
        q = aqk @ p["w_qkv"][:P].T + p["b_qkv"][:P]
        k = aqk @ p["w_qkv"][P:2 * P].T + p["b_qkv"][P:2 * P]
        v_raw = m["a_v"](a) @ p["w_qkv"][2 * P:].T + p["b_qkv"][2 * P:]
        qs, ks, v = m["q_s"](q), m["k_s"](k), m["v"](v_raw)
        c = np.zeros((B, S, P))
        lse = np.zeros((B, shape.n_heads, S))
        for b in range(B):
            for n in range(shape.n_heads):
                sl = slice(n * d, (n + 1) * d)
                s_ = np.where(mask, qs[b, :, sl] @ ks[b, :, sl].T * scale, -np.inf)
                mx = s_.max(1, keepdims=True)
                e = np.where(mask, np.exp(s_ - mx), 0.0)
                den = e.sum(1, keepdims=True)
                lse[b, n] = (mx + np.log(den))[:, 0]
                c[b, :, sl] = (m["p"](e) @ v[b, :, sl]) / den
        x1 = h + m["c"](c) @ p["w_o"].T + p["b_o"]
        a2_raw, xh2, r2 = orc.layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], shape.ln_eps)
        u = m["u"](m["a2"](a2_raw) @ p["w_fc1"].T + p["b_fc1"])
        g = m["g"](orc.gelu(u, shape.gelu))
        y = x1 + g @ p["w_fc2"].T + p["b_fc2"]
        if l == L - 1:
            y = m["yout"](y)
        saved.append(dict(a_w=m["a_w"](a), xh1=xh1, r1=r1, qs=qs, ks=ks, qg=m["q_g"](q), kg=m["k_g"](k),
                          vg=m["v_g"](v_raw), c_delta=m["c_delta"](c), c_w=m["c_w"](c), lse=lse,
                          a2_w=m["a2_w"](a2_raw), xh2=xh2, r2=r2, u=u, g=g))
        h = y
    grads = orc.zero_grads(params)
    flat = lambda t: t.reshape(-1, t.shape[-1])
    dcur = np.asarray(dy, np.float64)
    for l in range(L - 1, -1, -1):
        p, sv, G = params[l], saved[l], grads[l]
        dU = m["dU"]((dcur @ p["w_fc2"]) * orc.gelu_grad(sv["u"], shape.gelu))
        G["w_fc2"] += flat(dcur).T @ flat(sv["g"])
        G["b_fc2"] += flat(dcur).sum(0)
        dA2 = m["dA2"](dU @ p["w_fc1"])
        G["w_fc1"] += flat(dU).T @ flat(sv["a2_w"])
        G["b_fc1"] += flat(dU).sum(0)
        dln, dgam, dbet = orc.layernorm_bwd(dA2, sv["xh2"], sv["r2"], p["ln2_g"])
        G["ln2_g"] += dgam
        G["ln2_b"] += dbet
        dX1 = m["dX1"](dcur + dln)
        dC = m["dC"](dX1 @ p["w_o"])
        G["w_o"] += flat(dX1).T @ flat(sv["c_w"])
        G["b_o"] += flat(dX1).sum(0)
        dQ, dK, dV = np.zeros((B, S, P)), np.zeros((B, S, P)), np.zeros((B, S, P))
        for b in range(B):
            for n in range(shape.n_heads):
                sl = slice(n * d, (n + 1) * d)
                do = dC[b, :, sl]
                delta = (do * sv["c_delta"][b, :, sl]).sum(1, keepdims=True)
                s_ = sv["qs"][b, :, sl] @ sv["ks"][b, :, sl].T * scale
                pr = m["pb"](np.where(mask, np.exp(np.where(mask, s_, 0.0) - sv["lse"][b, n][:, None]), 0.0))
                ds = m["dS"](pr * (do @ sv["vg"][b, :, sl].T - delta))
                dQ[b, :, sl] = ds @ sv["kg"][b, :, sl] * scale
                dK[b, :, sl] = ds.T @ sv["qg"][b, :, sl] * scale
                dV[b, :, sl] = pr.T @ do
        dQKV = np.concatenate([m["dQ"](dQ), m["dK"](dK), m["dV"](dV)], axis=-1)
        dA = m["dA"](dQKV @ p["w_qkv"])
        G["w_qkv"] += flat(dQKV).T @ flat(sv["a_w"])
        G["b_qkv"] += flat(dQKV).sum(0)
        dln, dgam, dbet = orc.layernorm_bwd(dA, sv["xh1"], sv["r1"], p["ln1_g"])
        G["ln1_g"] += dgam
        G["ln1_b"] += dbet
        dcur = m["dX"](dX1 + dln)
    return h, dcur, grads


def max_norm_errors(got, ref):
    """{tensor: max|got-ref| / max|ref|} over y, dx and every non-zero gradient tensor."""
    err = lambda a, b: float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-300))
    out = {"y": err(got[0], ref[0]), "dx": err(got[1], ref[1])}
    for l, (ga, gb) in enumerate(zip(got[2], ref[2])):
        for k in gb:
            if np.any(gb[k]):
                out[f"L{l}.{k}"] = err(ga[k], gb[k])
    return out


def tp_share_inputs(seq):
    """The tensor-parallel-share workload cut to `seq` tokens, as fp64 arrays."""
    s = synth.WORKLOADS[4].with_(seq=seq)
    params = [{k: v.astype(np.float64) for k, v in p.items()} for p in synth.make_params(s, 0)]
    return s, synth.make_x(s, 0).astype(np.float64), synth.make_dy(s, 0).astype(np.float64), params


CASES = {
    "bf16 everywhere (plain bf16 stage)": {},
    "exact logit path (a for q/k, q, k)": dict(a_qk="exact", q_s="exact", k_s="exact"),
    "split-bf16 logit path": dict(a_qk="split", q_s="split", k_s="split"),
    "fp16 attention block (a, q, k, v, p, c)": dict(a_qk="fp16", a_v="fp16", q_s="fp16", k_s="fp16", v="fp16",
                                                    p="fp16", c="fp16", c_delta="fp16"),
    "fp16 forward activations (cfg.fwd_fp16)": FWD_FP16,
    "exact forward activations": {k: "exact" for k in FWD_FP16},
}


def main():
    seq = int(sys.argv[1]) if len(sys.argv) > 1 else 512
    s, x, dy, params = tp_share_inputs(seq)
    ref = orc.stage_fwd_bwd(x, dy, params, s.n_heads, s.head_dim, s.ln_eps, s.gelu)
    print(f"{s.name} at seq {seq}: tensor-max-normalised errors of the emulated stage against the oracle")
    for name, roles in CASES.items():
        t0 = time.time()
        e = max_norm_errors(emulate(s, x, dy, params, roles), ref)
        worst = sorted(e, key=e.get, reverse=True)[:3]
        print(f"  {name:44s} max {max(e.values()):.2e}  over 2e-2: {sum(v > 2e-2 for v in e.values()):2d}   "
              + " ".join(f"{k}={e[k]:.1e}" for k in worst) + f"   ({time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    main()
