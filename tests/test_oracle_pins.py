"""Pins for the CPU oracle: each test ties oracle/gpt_stage_oracle.py to
something other than itself -- finite differences, closed forms, invariants,
brute force with explicit index loops, and a rebuild of the layer from PyTorch
CPU fp64 primitives differentiated by autograd.  The paper prints no numeric
example of the stage computation (its section 4.1 and 5.2 only name the
forward and backward phases), so all pins are mathematical.
"""
import math

import numpy as np
import pytest
import torch

from oracle import gpt_stage_oracle as orc
from paper_2507_19845_amd import synth

TINY = synth.StageShape("pin_tiny", n_layers=2, hidden=16, n_heads=2, head_dim=8, ffn=32,
                        seq=8, batch=2, dtype="fp32", w_std=0.3, out_std=0.3,
                        bias_std=0.2, ln_jitter=0.2)
# attention width P != hidden (the tensor-parallel-share shape)
TINY_TP = TINY.with_(name="pin_tiny_tp", hidden=24, n_heads=2, head_dim=4, ffn=20)


def _p64(params):
    return [{k: v.astype(np.float64) for k, v in p.items()} for p in params]


def _setup(shape, seed=0):
    params = _p64(synth.make_params(shape, seed))
    x = synth.make_x(shape, seed).astype(np.float64)
    dy = synth.make_dy(shape, seed).astype(np.float64)
    return params, x, dy


def _loss(shape, params, x, dy, variant):
    y, _ = orc.stage_fwd(x, params, shape.n_heads, shape.head_dim, shape.ln_eps, variant)
    return float((y * dy).sum())


# ---------------------------------------------------------------- gradients ---
@pytest.mark.parametrize("shape", [TINY, TINY_TP], ids=lambda s: s.name)
@pytest.mark.parametrize("variant", ["tanh", "erf"])
def test_finite_differences_every_tensor(shape, variant):
    """<grad, v> == (l(theta+hv) - l(theta-hv)) / 2h for l = sum(y*dy), for x and
    every parameter tensor, along random directions."""
    params, x, dy = _setup(shape)
    _, dx, grads = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim,
                                     shape.ln_eps, variant)
    h = 1e-5
    rng = np.random.default_rng(1)

    def check(get, set_, grad, what):
        base = get().copy()
        for _ in range(3):
            v = rng.standard_normal(base.shape)
            set_(base + h * v); lp = _loss(shape, params, get_x(), dy, variant)
            set_(base - h * v); lm = _loss(shape, params, get_x(), dy, variant)
            set_(base)
            fd, an = (lp - lm) / (2 * h), float((grad * v).sum())
            assert abs(fd - an) <= 1e-7 * max(1.0, abs(an)), (what, fd, an)

    xbox = [x]
    get_x = lambda: xbox[0]
    check(lambda: xbox[0], lambda v: xbox.__setitem__(0, v), dx, "x")
    for l, p in enumerate(params):
        for name in orc.PARAM_NAMES:
            check(lambda: p[name], lambda v, p=p, name=name: p.__setitem__(name, v),
                  grads[l][name], f"layer{l}.{name}")


def test_finite_differences_single_coordinates():
    """Every coordinate of the small tensors (biases, LN parameters) and a sample
    of coordinates of x and of the weights."""
    shape, variant = TINY.with_(n_layers=1), "tanh"
    params, x, dy = _setup(shape, seed=3)
    _, dx, grads = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim,
                                     shape.ln_eps, variant)
    h = 1e-5
    rng = np.random.default_rng(2)
    p = params[0]
    for name in orc.PARAM_NAMES:
        flat = p[name].reshape(-1)
        idxs = range(flat.size) if flat.size <= 64 else rng.choice(flat.size, 24, replace=False)
        for i in idxs:
            old = flat[i]
            flat[i] = old + h; lp = _loss(shape, params, x, dy, variant)
            flat[i] = old - h; lm = _loss(shape, params, x, dy, variant)
            flat[i] = old
            an = grads[0][name].reshape(-1)[i]
            assert abs((lp - lm) / (2 * h) - an) <= 2e-7 * max(1.0, abs(an)), (name, i)
    xf = x.reshape(-1)
    for i in rng.choice(xf.size, 24, replace=False):
        old = xf[i]
        xf[i] = old + h; lp = _loss(shape, params, x, dy, variant)
        xf[i] = old - h; lm = _loss(shape, params, x, dy, variant)
        xf[i] = old
        an = dx.reshape(-1)[i]
        assert abs((lp - lm) / (2 * h) - an) <= 2e-7 * max(1.0, abs(an))


def _torch_layer(x, p, n_heads, d, eps, variant):
    """The same layer from PyTorch CPU fp64 library routines (no oracle code)."""
    F = torch.nn.functional
    H = x.shape[-1]
    P = n_heads * d
    a = F.layer_norm(x, (H,), p["ln1_g"], p["ln1_b"], eps)
    qkv = F.linear(a, p["w_qkv"], p["b_qkv"])
    B, S, _ = qkv.shape
    q, k, v = (t.reshape(B, S, n_heads, d).transpose(1, 2) for t in qkv.split(P, dim=-1))
    mask = torch.full((S, S), float("-inf"), dtype=x.dtype).triu(1)
    prob = torch.softmax(q @ k.transpose(-1, -2) / math.sqrt(d) + mask, dim=-1)
    c = (prob @ v).transpose(1, 2).reshape(B, S, P)
    x1 = x + F.linear(c, p["w_o"], p["b_o"])
    a2 = F.layer_norm(x1, (H,), p["ln2_g"], p["ln2_b"], eps)
    g = F.gelu(F.linear(a2, p["w_fc1"], p["b_fc1"]),
               approximate="tanh" if variant == "tanh" else "none")
    return x1 + F.linear(g, p["w_fc2"], p["b_fc2"])


@pytest.mark.parametrize("shape,variant", [
    (synth.WORKLOADS[0].with_(bias_std=0.02, ln_jitter=0.1), "tanh"),
    (synth.WORKLOADS[0].with_(bias_std=0.02, ln_jitter=0.1), "erf"),
    (synth.WORKLOADS[1].with_(n_layers=1, seq=128, batch=2, dtype="fp32", bias_std=0.02), "tanh"),
    (TINY_TP, "tanh"),
], ids=["w1_tanh", "w1_erf", "w2_cut", "tp"])
def test_against_autograd_rebuild(shape, variant):
    params, x, dy = _setup(shape)
    y, dx, grads = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim,
                                     shape.ln_eps, variant)
    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
          for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    h = tx
    for p in tp:
        h = _torch_layer(h, p, shape.n_heads, shape.head_dim, shape.ln_eps, variant)
    (h * torch.tensor(dy)).sum().backward()

    def rel(a, b):
        return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)

    assert rel(y, h.detach().numpy()) < 1e-10
    assert rel(dx, tx.grad.numpy()) < 1e-10
    for l, p in enumerate(tp):
        for name in orc.PARAM_NAMES:
            assert rel(grads[l][name], p[name].grad.numpy()) < 1e-10, (l, name)


# ---------------------------------------------------------------- attention ---
def test_softmax_rows_sum_to_one_and_upper_triangle_is_zero():
    rng = np.random.default_rng(0)
    q, k = rng.standard_normal((33, 8)) * 3, rng.standard_normal((33, 8)) * 3
    p = orc.causal_softmax(q, k)
    assert np.abs(p.sum(axis=1) - 1.0).max() < 1e-14
    assert np.all(np.triu(p, 1) == 0.0)
    assert np.all(p[np.tril_indices(33)] > 0.0)


def test_attention_brute_force_loops():
    """Explicit index loops (no matrix products) on a tiny case."""
    rng = np.random.default_rng(5)
    B, S, a, d = 2, 5, 3, 4
    P = a * d
    qkv = rng.standard_normal((B, S, 3 * P))
    got = orc.attention_fwd(qkv, a, d)
    want = np.zeros((B, S, P))
    for b in range(B):
        for n in range(a):
            for i in range(S):
                sc = [sum(qkv[b, i, n * d + c] * qkv[b, j, P + n * d + c] for c in range(d)) / math.sqrt(d)
                      for j in range(i + 1)]
                m = max(sc)
                e = [math.exp(s - m) for s in sc]
                z = sum(e)
                for c in range(d):
                    want[b, i, n * d + c] = sum(e[j] / z * qkv[b, j, 2 * P + n * d + c] for j in range(i + 1))
    assert np.abs(got - want).max() < 1e-14


def test_attention_closed_forms():
    rng = np.random.default_rng(6)
    B, S, a, d = 2, 9, 2, 4
    P = a * d
    qkv = rng.standard_normal((B, S, 3 * P))
    out = orc.attention_fwd(qkv, a, d)
    # row 0 attends only to itself
    assert np.array_equal(out[:, 0, :], qkv[:, 0, 2 * P:])
    # zero queries -> uniform probabilities 1/(i+1) -> prefix mean of V
    z = qkv.copy(); z[:, :, :P] = 0.0
    out = orc.attention_fwd(z, a, d)
    prefix_mean = np.cumsum(qkv[:, :, 2 * P:], axis=1) / np.arange(1, S + 1)[None, :, None]
    assert np.abs(out - prefix_mean).max() < 1e-14
    # S = 1: identity on V
    one = rng.standard_normal((3, 1, 3 * P))
    assert np.array_equal(orc.attention_fwd(one, a, d), one[:, :, 2 * P:])


def test_attention_score_gradient_rows_sum_to_zero():
    """All keys equal => scores constant along a row => softmax is independent of
    q, so dQ = (sum_j dS_ij) k / sqrt(d) must vanish: pins sum_j dS_ij = 0."""
    rng = np.random.default_rng(7)
    S, a, d = 7, 2, 4
    P = a * d
    qkv = rng.standard_normal((1, S, 3 * P))
    qkv[:, :, P:2 * P] = qkv[:, :1, P:2 * P]
    dq = orc.attention_bwd(qkv, rng.standard_normal((1, S, P)), a, d)[:, :, :P]
    assert np.abs(dq).max() < 1e-14


# --------------------------------------------------------------- whole stage ---
def test_zero_weight_identity_residual():
    """All W = 0 and b = 0: y = x and dx = dy exactly; every parameter gradient
    is zero except db_o = db_fc2 = sum_t dy_t."""
    shape = TINY
    params, x, dy = _setup(shape)
    for p in params:
        for k in p:
            if k.startswith("w_") or k.startswith("b_"):
                p[k][...] = 0.0
    y, dx, grads = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim)
    assert np.array_equal(y, x)
    assert np.array_equal(dx, dy)
    colsum = dy.reshape(-1, shape.hidden).sum(axis=0)
    for g in grads:
        for k, v in g.items():
            if k in ("b_o", "b_fc2"):
                assert np.abs(v - colsum).max() < 1e-13
            else:
                assert np.all(v == 0.0), k


def test_causality_and_batch_independence():
    shape = TINY
    params, x, dy = _setup(shape)
    y, dx, _ = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim)
    t = 5
    x2 = x.copy(); x2[0, t:, :] += 1.0
    y2, _ = orc.stage_fwd(x2, params, shape.n_heads, shape.head_dim)
    assert np.array_equal(y2[0, :t], y[0, :t])          # earlier tokens untouched, bit for bit
    assert not np.array_equal(y2[0, t:], y[0, t:])
    assert np.array_equal(y2[1], y[1])                   # other batch element untouched
    dy2 = dy.copy(); dy2[0, :t, :] += 1.0
    _, dx2, _ = orc.stage_fwd_bwd(x, dy2, params, shape.n_heads, shape.head_dim)
    assert np.array_equal(dx2[0, t:], dx[0, t:])         # dx_t sees only dy at t' >= t
    assert np.array_equal(dx2[1], dx[1])


def test_backward_is_linear_in_dy():
    shape = TINY
    params, x, dy = _setup(shape)
    dy_b = synth.make_dy(shape, seed=9).astype(np.float64)
    _, dx_a, g_a = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim)
    _, dx_b, g_b = orc.stage_fwd_bwd(x, dy_b, params, shape.n_heads, shape.head_dim)
    _, dx_c, g_c = orc.stage_fwd_bwd(x, 2.0 * dy - 3.0 * dy_b, params, shape.n_heads, shape.head_dim)
    assert np.abs(dx_c - (2 * dx_a - 3 * dx_b)).max() < 1e-12
    for ga, gb, gc in zip(g_a, g_b, g_c):
        for k in ga:
            assert np.abs(gc[k] - (2 * ga[k] - 3 * gb[k])).max() < 1e-11 * max(1.0, np.abs(gc[k]).max())


def test_microbatch_accumulation_equals_one_big_batch():
    """Gradients of 4 micro-batches of size 1 accumulated into one buffer equal
    those of one batch of size 4; y and dx are the concatenation."""
    shape = TINY.with_(batch=4)
    params, x, dy = _setup(shape)
    y, dx, g_big = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim)
    acc = orc.zero_grads(params)
    for b in range(4):
        yb, dxb, _ = orc.stage_fwd_bwd(x[b:b + 1], dy[b:b + 1], params, shape.n_heads,
                                       shape.head_dim, grads=acc)
        assert np.abs(yb - y[b:b + 1]).max() < 1e-13
        assert np.abs(dxb - dx[b:b + 1]).max() < 1e-13
    for ga, gb in zip(acc, g_big):
        for k in ga:
            assert np.abs(ga[k] - gb[k]).max() < 1e-12 * max(1.0, np.abs(gb[k]).max())


def test_tensor_parallel_shares_sum_to_the_full_branch():
    """Splitting heads (and MLP columns) into shards and summing the shards'
    un-reduced partial products reproduces the full branch: pins the head and
    column indexing used when attention width != hidden."""
    shape = TINY.with_(n_heads=4, head_dim=4, hidden=16, ffn=32)
    params, x, _ = _setup(shape)
    p = params[0]
    P, d = shape.attn_width, shape.head_dim
    full = orc.attn_branch_fwd(x, p, shape.n_heads, d)
    part = np.zeros_like(full)
    for r in range(2):
        heads = slice(r * 2 * d, (r + 1) * 2 * d)
        rows = np.r_[np.arange(P)[heads], P + np.arange(P)[heads], 2 * P + np.arange(P)[heads]]
        shard = dict(w_qkv=p["w_qkv"][rows], b_qkv=p["b_qkv"][rows], w_o=p["w_o"][:, heads])
        part += orc.attn_branch_fwd(x, shard, 2, d)
    assert np.abs(part - full).max() < 1e-13
    full = orc.mlp_branch_fwd(x, p)
    part = np.zeros_like(full)
    for r in range(2):
        cols = slice(r * 16, (r + 1) * 16)
        shard = dict(w_fc1=p["w_fc1"][cols], b_fc1=p["b_fc1"][cols], w_fc2=p["w_fc2"][:, cols])
        part += orc.mlp_branch_fwd(x, shard)
    assert np.abs(part - full).max() < 1e-13


# ---------------------------------------------------------------- LayerNorm ---
def test_layernorm_invariants():
    rng = np.random.default_rng(8)
    H, eps = 48, 1e-5
    x = rng.standard_normal((3, 7, H)) * 2 + 0.7
    gamma, beta = rng.standard_normal(H), rng.standard_normal(H)
    out, xhat, r = orc.layernorm_fwd(x, gamma, beta, eps)
    var = x.var(axis=-1, keepdims=True)                   # numpy's biased variance
    assert np.abs(xhat.sum(axis=-1)).max() < 1e-12
    assert np.abs((xhat ** 2).mean(axis=-1, keepdims=True) - var / (var + eps)).max() < 1e-12
    assert np.abs(out - (xhat * gamma + beta)).max() == 0.0
    dout = rng.standard_normal(x.shape)
    dx, dgam, dbet = orc.layernorm_bwd(dout, xhat, r, gamma)
    assert np.abs(dx.sum(axis=-1)).max() < 1e-12           # orthogonal to 1
    # <dx, xhat> = r <g, xhat> eps/(var+eps): orthogonal to xhat up to the eps term
    g = dout * gamma
    want = (r * (g * xhat).sum(axis=-1, keepdims=True) * eps / (var + eps))[..., 0]
    assert np.abs((dx * xhat).sum(axis=-1) - want).max() < 1e-12
    dx0, _, _ = orc.layernorm_bwd(dout, *orc.layernorm_fwd(x, gamma, beta, 0.0)[1:], gamma)
    assert np.abs((dx0 * orc.layernorm_fwd(x, gamma, beta, 0.0)[1]).sum(axis=-1)).max() < 1e-12
    assert np.abs(dbet - dout.reshape(-1, H).sum(0)).max() < 1e-12
    # constant row, gamma = 1, beta = 0 -> output 0
    out, _, _ = orc.layernorm_fwd(np.full((2, H), 3.25), np.ones(H), np.zeros(H), eps)
    assert np.all(out == 0.0)
    # scale invariance up to eps: LN(c x) == LN(x) as eps -> 0
    o1, _, _ = orc.layernorm_fwd(x, gamma, beta, 0.0)
    o2, _, _ = orc.layernorm_fwd(5.0 * x, gamma, beta, 0.0)
    assert np.abs(o1 - o2).max() < 1e-12


# --------------------------------------------------------------------- GeLU ---
def test_gelu_values_and_identities():
    from scipy.stats import norm
    u = np.linspace(-8, 8, 160001)
    for variant in ("tanh", "erf"):
        assert orc.gelu(0.0, variant) == 0.0
        assert np.abs(orc.gelu(u, variant) - orc.gelu(-u, variant) - u).max() < 1e-14
        h = 1e-6
        fd = (orc.gelu(u + h, variant) - orc.gelu(u - h, variant)) / (2 * h)
        assert np.abs(fd - orc.gelu_grad(u, variant)).max() < 1e-8
    # erf form is u * Phi(u), Phi = standard normal cdf (library routine)
    assert np.abs(orc.gelu(u, "erf") - u * norm.cdf(u)).max() < 1e-14
    # textbook constants: gelu(1) = Phi(1) = 0.8413447...; tanh form 0.8411920...
    assert abs(float(orc.gelu(1.0, "erf")) - 0.8413447460685429) < 1e-15
    assert abs(float(orc.gelu(1.0, "tanh")) - 0.8411919906082768) < 1e-15
    # the two forms differ by at most ~4.73e-4, reached near |u| = 2.70
    diff = np.abs(orc.gelu(u, "tanh") - orc.gelu(u, "erf"))
    assert 4.72e-4 < diff.max() < 4.74e-4
    assert abs(abs(u[diff.argmax()]) - 2.70) < 0.01


# ----------------------------------------------- the pins have teeth (CPU only) ---
@pytest.mark.parametrize("mutation", ["drop_residual", "wrong_sign_ln", "transposed_dk", "no_scale"])
def test_planted_mistakes_are_caught(monkeypatch, mutation):
    """Plant a plausible mistake in the oracle and check the finite-difference pin
    rejects it (so the pin would catch the same mistake made for real)."""
    shape, variant = TINY.with_(n_layers=1), "tanh"
    params, x, dy = _setup(shape)
    if mutation == "drop_residual":
        good = orc.layernorm_bwd
        calls = []

        def bad(dout, xhat, r, gamma):
            dx, a, b = good(dout, xhat, r, gamma)
            calls.append(1)
            return (dx * 0.0 if len(calls) == 1 else dx), a, b
        monkeypatch.setattr(orc, "layernorm_bwd", bad)
    elif mutation == "wrong_sign_ln":
        def bad(dout, xhat, r, gamma):
            g = dout * gamma
            dx = r * (g - g.mean(-1, keepdims=True) + xhat * (g * xhat).mean(-1, keepdims=True))
            red = tuple(range(dout.ndim - 1))
            return dx, (dout * xhat).sum(axis=red), dout.sum(axis=red)
        monkeypatch.setattr(orc, "layernorm_bwd", bad)
    elif mutation == "transposed_dk":
        good = orc.attention_bwd

        def bad(qkv, dout, a, d):
            out = good(qkv, dout, a, d)
            P = a * d
            out[:, :, P:2 * P] = out[:, ::-1, P:2 * P]
            return out
        monkeypatch.setattr(orc, "attention_bwd", bad)
    elif mutation == "no_scale":
        good = orc.attention_bwd
        monkeypatch.setattr(orc, "attention_bwd",
                            lambda qkv, dout, a, d: good(qkv, dout, a, d) * math.sqrt(d))
    _, dx, _ = orc.stage_fwd_bwd(x, dy, params, shape.n_heads, shape.head_dim, shape.ln_eps, variant)
    h = 1e-5
    v = np.random.default_rng(0).standard_normal(x.shape)
    fd = (_loss(shape, params, x + h * v, dy, variant) - _loss(shape, params, x - h * v, dy, variant)) / (2 * h)
    assert abs(fd - float((dx * v).sum())) > 1e-4 * max(1.0, abs(fd))
