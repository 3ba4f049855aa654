"""Shared helpers of the GPU parity tests: run a workload through the C-ABI and
through the oracle on the same seeded inputs and compare tensor by tensor."""
import numpy as np
import torch

from oracle import gpt_stage_oracle as orc
from paper_2507_19845_amd import binding as B
from paper_2507_19845_amd import harness, synth

# tensor-max-normalised max error allowed per storage type
TOL = {"fp32": 1e-4, "bf16": 2e-2}


def max_norm_err(got, ref) -> float:
    """max|got-ref| / max|ref| over one tensor (ref all-zero: absolute error)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def p64(params):
    return [{k: v.astype(np.float64) for k, v in p.items()} for p in params]


def gpu_run(shape, params, xs, dys, decoupled=False, bufs=None, trace=None, split_wgrad=False):
    """Returns (ys, dxs, grads) as float64 numpy, parameter gradients accumulated
    over the given micro-batches.  trace: tracer handle attached to the stage calls."""
    n = len(xs)
    if bufs is None:
        bufs = B.StageBuffers(shape, n_stash=n if decoupled else 1)
        bufs.load_params(params)
    bufs.trace = trace
    bufs.dparams.zero_()
    dxs_in = [B.to_device(x, shape.dtype) for x in xs]
    dys_in = [B.to_device(d, shape.dtype) for d in dys]
    ys = [bufs.act() for _ in range(n)]
    dxs = [bufs.act() for _ in range(n)]
    runner = harness.StageRunner(bufs)
    if decoupled:
        runner.decoupled(dxs_in, dys_in, ys, dxs, split_wgrad=split_wgrad)
    else:
        runner.coupled(dxs_in, dys_in, ys, dxs)
    torch.cuda.synchronize()
    bufs.trace = None
    return [B.to_host(y) for y in ys], [B.to_host(d) for d in dxs], bufs.read_grads()


def oracle_run(shape, params, xs, dys):
    pp = p64(params)
    grads = orc.zero_grads(pp)
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        y, dx, _ = orc.stage_fwd_bwd(x.astype(np.float64), dy.astype(np.float64), pp, shape.n_heads,
                                     shape.head_dim, shape.ln_eps, shape.gelu, grads=grads)
        ys.append(y)
        dxs.append(dx)
    return ys, dxs, grads


def compare(shape, got, ref, tol=None):
    """Assert every tensor within tolerance; returns {name: err}."""
    tol = TOL[shape.dtype] if tol is None else tol
    errs = {}
    gy, gdx, gg = got
    ry, rdx, rg = ref
    for i, (a, b) in enumerate(zip(gy, ry)):
        errs[f"y[{i}]"] = max_norm_err(a, b)
    for i, (a, b) in enumerate(zip(gdx, rdx)):
        errs[f"dx[{i}]"] = max_norm_err(a, b)
    for l, (a, b) in enumerate(zip(gg, rg)):
        for k in b:
            errs[f"L{l}.{k}"] = max_norm_err(a[k], b[k])
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, f"{shape.name}: over tolerance {tol}: {bad}"
    return errs
