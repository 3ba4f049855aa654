"""CPU fp64 oracle for the forward and backward pass of one GPT pipeline stage.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP library is checked against.  Nothing in the product path may import it;
it imports nothing from the product either.  It shares no code, constants or
helpers with the HIP kernels.

What it computes.  The paper reschedules two phases of a pipeline stage -- the
"forward phase" and the "backward phase (gradient computation)" of section 4.1
(MegaFBD, motivation), one task of the (model chunk, micro-batch) matrix of
section 5.2 (MegaDPP, parallel scheduler) -- but takes the layer mathematics
from the GPT/Megatron-LM layer it builds on (section 2.2-2.3, citing the
Transformer).  The stage is therefore L pre-LayerNorm GPT decoder layers and
the result has a plain textbook definition, written out below with explicit
formulas; `@` (a library matrix product) is the only library primitive used as
a step.  There is no tiling, no online softmax, no fusion: attention
materialises each head's S x S probability matrix.

Readings taken where the paper is silent (it defines none of these):
  * a stage = exactly L decoder layers; no embedding, final norm, head or loss;
  * every linear layer has a bias; no dropout;
  * LayerNorm uses the biased variance and eps inside the square root;
  * softmax scale is 1/sqrt(head_dim); positions j > i get probability exactly 0;
  * GeLU is the tanh approximation unless gelu="erf";
  * fused QKV weight rows are [all Q heads | all K heads | all V heads];
  * parameter gradients ACCUMULATE into the buffers handed in (summing over
    micro-batches as section 5.2's breadth-first order requires).

Every function here is pinned by tests/test_oracle_pins.py (finite
differences, closed forms, invariants, and an independent autograd rebuild);
nothing is "parity unpinned".

Array conventions: float64 numpy arrays; activations [B, S, width]; weights
[out, in]; a layer's parameters are a dict keyed by the names in PARAM_NAMES.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf

PARAM_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)

_KAPPA = math.sqrt(2.0 / math.pi)
_C3 = 0.044715


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


# ------------------------------------------------------------- LayerNorm ------
def layernorm_fwd(x, gamma, beta, eps: float):
    """Per token (last axis):  mu = mean(x), var = mean((x-mu)^2) (biased),
    r = 1/sqrt(var+eps), xhat = (x-mu) r, out = xhat*gamma + beta.
    Returns (out, xhat, r) with r shaped [..., 1]."""
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * r
    return xhat * _f64(gamma) + _f64(beta), xhat, r


def layernorm_bwd(dout, xhat, r, gamma):
    """Reverse of layernorm_fwd.  With g = dout*gamma:
        dx     = r * (g - mean(g) - xhat * mean(g*xhat))     (means over the row)
        dgamma = sum_tokens dout*xhat ,  dbeta = sum_tokens dout.
    Returns (dx, dgamma, dbeta)."""
    dout = _f64(dout)
    g = dout * _f64(gamma)
    dx = r * (g - g.mean(axis=-1, keepdims=True)
              - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dout.ndim - 1))
    return dx, (dout * xhat).sum(axis=red), dout.sum(axis=red)


# ------------------------------------------------------------------ GeLU ------
def gelu(u, variant: str = "tanh"):
    u = _f64(u)
    if variant == "tanh":
        return 0.5 * u * (1.0 + np.tanh(_KAPPA * (u + _C3 * u ** 3)))
    if variant == "erf":
        return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))
    raise ValueError(variant)


def gelu_grad(u, variant: str = "tanh"):
    """d gelu / du."""
    u = _f64(u)
    if variant == "tanh":
        t = np.tanh(_KAPPA * (u + _C3 * u ** 3))
        return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _KAPPA * (1.0 + 3.0 * _C3 * u * u)
    if variant == "erf":
        cdf = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
        return cdf + u * pdf
    raise ValueError(variant)


# ------------------------------------------------------------- attention ------
def causal_softmax(q, k):
    """P[i, j] for one head.  q, k: [S, d].
    s_ij = q_i . k_j / sqrt(d);  P_ij = exp(s_ij - m_i) / sum_{l<=i} exp(s_il - m_i)
    for j <= i with m_i = max_{l<=i} s_il, and P_ij = 0 exactly for j > i."""
    S, d = q.shape
    s = (q @ k.T) / math.sqrt(d)
    allowed = np.tril(np.ones((S, S), dtype=bool))
    s = np.where(allowed, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.where(allowed, np.exp(s - m), 0.0)
    return e / e.sum(axis=1, keepdims=True)


def attention_fwd(qkv, n_heads: int, head_dim: int):
    """qkv: [B, S, 3P] laid out [Q | K | V], head n = columns n*d .. (n+1)*d-1 of
    each block.  Returns the concatenated head outputs C: [B, S, P]."""
    qkv = _f64(qkv)
    B, S, _ = qkv.shape
    P = n_heads * head_dim
    out = np.zeros((B, S, P))
    for b in range(B):
        for n in range(n_heads):
            c0, c1 = n * head_dim, (n + 1) * head_dim
            q, k, v = qkv[b, :, c0:c1], qkv[b, :, P + c0:P + c1], qkv[b, :, 2 * P + c0:2 * P + c1]
            out[b, :, c0:c1] = causal_softmax(q, k) @ v
    return out


def attention_bwd(qkv, dout, n_heads: int, head_dim: int):
    """Gradient of attention_fwd w.r.t. qkv.  Per head, with P recomputed from
    its definition:  dV = P^T dO;  dP = dO V^T;  dS_ij = P_ij (dP_ij - sum_l P_il dP_il);
    dQ = dS K / sqrt(d);  dK = dS^T Q / sqrt(d)."""
    qkv, dout = _f64(qkv), _f64(dout)
    B, S, _ = qkv.shape
    P = n_heads * head_dim
    dqkv = np.zeros_like(qkv)
    scale = 1.0 / math.sqrt(head_dim)
    for b in range(B):
        for n in range(n_heads):
            c0, c1 = n * head_dim, (n + 1) * head_dim
            q, k, v = qkv[b, :, c0:c1], qkv[b, :, P + c0:P + c1], qkv[b, :, 2 * P + c0:2 * P + c1]
            do = dout[b, :, c0:c1]
            p = causal_softmax(q, k)
            dp = do @ v.T
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dqkv[b, :, c0:c1] = (ds @ k) * scale
            dqkv[b, :, P + c0:P + c1] = (ds.T @ q) * scale
            dqkv[b, :, 2 * P + c0:2 * P + c1] = p.T @ do
    return dqkv


# ----------------------------------------------------------------- layer ------
def attn_branch_fwd(a, p, n_heads, head_dim):
    """The attention branch WITHOUT the residual: C(a) W_o^T (no b_o).  Used by
    the tensor-parallel-share consistency pin."""
    qkv = _f64(a) @ _f64(p["w_qkv"]).T + _f64(p["b_qkv"])
    return attention_fwd(qkv, n_heads, head_dim) @ _f64(p["w_o"]).T


def mlp_branch_fwd(a2, p, variant="tanh"):
    """The MLP branch WITHOUT residual and without b_fc2: gelu(a2 W1^T + b1) W2^T."""
    return gelu(_f64(a2) @ _f64(p["w_fc1"]).T + _f64(p["b_fc1"]), variant) @ _f64(p["w_fc2"]).T


def layer_fwd(x, p: Dict[str, np.ndarray], n_heads: int, head_dim: int,
              eps: float = 1e-5, variant: str = "tanh"):
    """One pre-LN decoder layer.  x: [B, S, H].  Returns (y, saved)."""
    x = _f64(x)
    a, xhat1, r1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = a @ _f64(p["w_qkv"]).T + _f64(p["b_qkv"])
    c = attention_fwd(qkv, n_heads, head_dim)
    x1 = x + c @ _f64(p["w_o"]).T + _f64(p["b_o"])
    a2, xhat2, r2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    u = a2 @ _f64(p["w_fc1"]).T + _f64(p["b_fc1"])
    g = gelu(u, variant)
    y = x1 + g @ _f64(p["w_fc2"]).T + _f64(p["b_fc2"])
    saved = dict(a=a, xhat1=xhat1, r1=r1, qkv=qkv, c=c, a2=a2, xhat2=xhat2, r2=r2, u=u, g=g)
    return y, saved


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_bwd(dy, p, saved, grads: Dict[str, np.ndarray], n_heads: int, head_dim: int,
              variant: str = "tanh"):
    """Reverse of layer_fwd.  Adds this call's parameter gradients INTO `grads`
    (float64 arrays of the parameter shapes) and returns dx."""
    dy = _f64(dy)
    # y = x1 + g W2^T + b2
    dg = dy @ _f64(p["w_fc2"])
    grads["w_fc2"] += _flat(dy).T @ _flat(saved["g"])
    grads["b_fc2"] += _flat(dy).sum(axis=0)
    # g = gelu(u);  u = a2 W1^T + b1
    du = dg * gelu_grad(saved["u"], variant)
    da2 = du @ _f64(p["w_fc1"])
    grads["w_fc1"] += _flat(du).T @ _flat(saved["a2"])
    grads["b_fc1"] += _flat(du).sum(axis=0)
    # a2 = LN2(x1);  x1 also feeds the residual
    dx1_ln, dgam, dbet = layernorm_bwd(da2, saved["xhat2"], saved["r2"], p["ln2_g"])
    grads["ln2_g"] += dgam
    grads["ln2_b"] += dbet
    dx1 = dy + dx1_ln
    # x1 = x + c Wo^T + bo
    dc = dx1 @ _f64(p["w_o"])
    grads["w_o"] += _flat(dx1).T @ _flat(saved["c"])
    grads["b_o"] += _flat(dx1).sum(axis=0)
    # c = attention(qkv);  qkv = a Wqkv^T + bqkv
    dqkv = attention_bwd(saved["qkv"], dc, n_heads, head_dim)
    da = dqkv @ _f64(p["w_qkv"])
    grads["w_qkv"] += _flat(dqkv).T @ _flat(saved["a"])
    grads["b_qkv"] += _flat(dqkv).sum(axis=0)
    # a = LN1(x);  x also feeds the residual
    dx_ln, dgam, dbet = layernorm_bwd(da, saved["xhat1"], saved["r1"], p["ln1_g"])
    grads["ln1_g"] += dgam
    grads["ln1_b"] += dbet
    return dx1 + dx_ln


# ----------------------------------------------------------------- stage ------
def zero_grads(params: List[Dict[str, np.ndarray]]) -> List[Dict[str, np.ndarray]]:
    return [{k: np.zeros(np.shape(v), dtype=np.float64) for k, v in p.items()} for p in params]


def stage_fwd(x, params: List[Dict[str, np.ndarray]], n_heads: int, head_dim: int,
              eps: float = 1e-5, variant: str = "tanh"):
    """Forward phase of the stage: layers applied in order.  Returns (y, stash);
    the stash (one entry per layer) is what the backward phase consumes."""
    stash = []
    h = _f64(x)
    for p in params:
        h, saved = layer_fwd(h, p, n_heads, head_dim, eps, variant)
        stash.append(saved)
    return h, stash


def stage_bwd(dy, params, stash, grads, n_heads: int, head_dim: int, variant: str = "tanh"):
    """Backward phase: layers in reverse order; parameter gradients accumulate
    into `grads`; returns dx = d(sum(y*dy))/dx."""
    d = _f64(dy)
    for p, saved, g in zip(reversed(params), reversed(stash), reversed(grads)):
        d = layer_bwd(d, p, saved, g, n_heads, head_dim, variant)
    return d


def stage_fwd_bwd(x, dy, params, n_heads, head_dim, eps=1e-5, variant="tanh",
                  grads: Optional[List[Dict[str, np.ndarray]]] = None):
    """Convenience: one micro-batch forward then backward.  Returns (y, dx, grads)."""
    if grads is None:
        grads = zero_grads(params)
    y, stash = stage_fwd(x, params, n_heads, head_dim, eps, variant)
    dx = stage_bwd(dy, params, stash, grads, n_heads, head_dim, variant)
    return y, dx, grads
