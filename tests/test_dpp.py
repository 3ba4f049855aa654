"""Traversal of the (micro-batch, chunk) task matrix (section 5.2, MegaDPP "parallel scheduler").

CPU part: the Python oracle of the three traversal orders is pinned to what the paper fixes
(figure 3: 8 chunks x 8 micro-batches = 64 tasks named "i-j"; row-wise vs column-wise order;
depth first releases activation memory soonest, breadth first completes a chunk's gradients
soonest) and to brute force on small matrices; the library's host-side planner must give the
same order, task for task.  GPU part: the driver runs several chunks through the decoupled
entry points and must reproduce the oracle of the whole layer stack, bit-identically across
policies."""
import itertools
import os

import numpy as np
import pytest

from oracle import dpp_oracle as dpo
from paper_2507_19845_amd import binding as B
from paper_2507_19845_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "dpp_task_matrix.txt")
POLICY = {"dfc": B.GPT_DPP_DFC, "bfc": B.GPT_DPP_BFC, "bfc_best_effort": B.GPT_DPP_BFC_BEST_EFFORT}


def _golden():
    kv = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            kv[k] = int(v)
    return kv


def test_figure3_matrix():
    g = _golden()
    C, M = g["chunks"], g["microbatches"]
    mat = dpo.task_matrix(C, M)
    assert sum(len(r) for r in mat) == g["tasks"] == 64
    assert mat[3][5] == "3-5"          # "i-j": micro-batch i on chunk j
    assert len({t for r in mat for t in r}) == 64
    # executing "along the micro-batch (row) or model-chunk (column) dimension":
    fwd = lambda order: [dpo.task_name(i, j) for ph, i, j in order if ph == "F"]
    assert fwd(dpo.depth_first(C, M)) == [t for row in mat for t in row]
    assert fwd(dpo.breadth_first(C, M)) == [mat[i][j] for j in range(C) for i in range(M)]


@pytest.mark.parametrize("C,M", [(1, 1), (1, 5), (4, 1), (2, 3), (8, 8), (3, 7)])
def test_orders_are_valid_and_have_the_stated_memory_behaviour(C, M):
    dfc, bfc = dpo.depth_first(C, M), dpo.breadth_first(C, M)
    assert dpo.dependencies_hold(dfc, C, M) and dpo.dependencies_hold(bfc, C, M)
    # depth first: one micro-batch in flight; breadth first: every stash alive at the turn
    assert dpo.peak_live_stash(dfc) == C
    assert dpo.peak_live_stash(bfc) == C * M
    # breadth first completes the LAST chunk's gradients after C*M forward + M backward tasks,
    # depth first only with the last micro-batch
    assert dpo.gradient_ready_position(bfc, C)[C - 1] == C * M + M - 1
    assert dpo.gradient_ready_position(dfc, C)[C - 1] == 2 * C * (M - 1) + C
    for cap in range(0, C * M + 3):
        be = dpo.best_effort_breadth_first(C, M, cap)
        assert dpo.dependencies_hold(be, C, M)
        peak = dpo.peak_live_stash(be)
        assert peak <= max(cap, C)                 # never above the allowance (one micro-batch minimum)
        assert peak > cap - C or peak == C * M     # and as breadth-first as the allowance permits
        if cap >= C * M:
            assert be == bfc
        if cap < 2 * C:
            assert be == dfc


def test_orders_against_brute_force():
    """On a 2x2 matrix enumerate every valid order: depth first has the smallest peak stash
    among all of them, breadth first the earliest completion of the last chunk's gradients."""
    C = M = 2
    tasks = [(p, i, j) for p in "FB" for i in range(M) for j in range(C)]
    valid = [o for o in itertools.permutations(tasks) if dpo.dependencies_hold(list(o), C, M)]
    assert len(valid) > 10
    assert dpo.peak_live_stash(dpo.depth_first(C, M)) == min(dpo.peak_live_stash(o) for o in valid)
    ready = lambda o: dpo.gradient_ready_position(o, C)[C - 1]
    assert ready(dpo.breadth_first(C, M)) == min(ready(o) for o in valid)


def test_planted_mistake_is_caught():
    bad = dpo.breadth_first(3, 2)
    k = bad.index(("B", 0, 2))
    bad[k], bad[k + 1] = ("B", 0, 1), bad[k]     # backward of chunk 1 before chunk 2
    assert not dpo.dependencies_hold(bad, 3, 2)


@pytest.mark.parametrize("C,M", [(1, 1), (4, 8), (8, 8), (3, 5)])
def test_library_plan_equals_oracle(C, M):
    ph = {B.GPT_DPP_FWD: "F", B.GPT_DPP_BWD: "B"}
    for name, pol in POLICY.items():
        for cap in ([0] if name != "bfc_best_effort" else [0, C, 2 * C, 2 * C + 1, C * M - 1, C * M, 10 * C * M]):
            got, peak = B.gpt_dpp_plan(pol, C, M, cap)
            ref = dpo.traversal(name, C, M, cap)
            assert [(ph[p], i, j) for p, i, j in got] == ref, (name, cap)
            assert peak == dpo.peak_live_stash(ref)


def test_library_plan_rejects_bad_arguments():
    with pytest.raises(B.GptStageError):
        B.gpt_dpp_plan(7, 2, 2, 0)
    with pytest.raises(B.GptStageError):
        B.gpt_dpp_plan(B.GPT_DPP_DFC, 0, 2, 0)
    arr = (B.gpt_dpp_task * 4)()
    assert B.lib().gpt_dpp_plan(B.GPT_DPP_DFC, 2, 2, 0, arr, 4, None) == B.GPTS_ENOMEM


# ---- GPU: the driver ---------------------------------------------------------------------
def _run_dpp(shape, C, M, policy, cap, params_np, pool_slots=None, expect_peak=None, weight_phase=False):
    import torch
    chunk_shape = shape.with_(n_layers=shape.n_layers // C)
    Lc = chunk_shape.n_layers
    cfg = B.make_cfg(chunk_shape)
    nparam = B.gpt_stage_param_count(cfg)
    ws = torch.empty(max(B.gpt_stage_workspace_bytes(cfg, 1), 256), dtype=torch.uint8, device="cuda")
    chunks, weights, dps = [], [], []
    for j in range(C):
        w = torch.empty(nparam, dtype=torch.bfloat16 if shape.dtype == "bf16" else torch.float32, device="cuda")
        for l in range(Lc):
            for tid, name in enumerate(synth.TENSOR_NAMES):
                off, n = B.gpt_stage_param_offset(cfg, l, tid)
                w[off:off + n].copy_(B.to_device(params_np[j * Lc + l][name].reshape(-1), shape.dtype))
        weights.append(w)
        dps.append(torch.zeros(nparam, dtype=torch.float32, device="cuda"))
        chunks.append(B.gpt_stage_params(cfg=cfg, weights=w.data_ptr(), workspace=ws.data_ptr(), prepared=None, trace=None))
    xs = [B.to_device(synth.make_x(shape, 0, m), shape.dtype) for m in range(M)]
    dys = [B.to_device(synth.make_dy(shape, 0, m), shape.dtype) for m in range(M)]
    ys = [torch.empty_like(x) for x in xs]
    dxs = [torch.empty_like(x) for x in xs]
    _, peak = B.gpt_dpp_plan(policy, C, M, cap)
    if pool_slots is not None:
        peak = expect_peak
    stash = torch.empty(B.gpt_dpp_stash_slot_bytes(chunks) * (pool_slots or peak), dtype=torch.uint8, device="cuda")
    act = torch.empty(B.gpt_dpp_act_slot_bytes(cfg) * (2 * M + 2), dtype=torch.uint8, device="cuda")
    grad_pool = None
    if weight_phase:     # one gradient-stash slot per micro-batch of a window (peak = n_chunks * window)
        grad_pool = torch.empty(B.gpt_dpp_grad_slot_bytes(chunks) * (peak // C), dtype=torch.uint8, device="cuda")
    rep = B.gpt_dpp_run(policy, chunks, xs, dys, ys, dxs, dps, stash, act, max_live_stash=cap, grad_pool=grad_pool)
    torch.cuda.synchronize()
    assert rep.n_tasks == 2 * C * M and rep.peak_live_stash == peak
    return ([B.to_host(t) for t in ys], [B.to_host(t) for t in dxs], [t.cpu().numpy() for t in dps], cfg, rep)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_dpp_driver_matches_oracle_and_policies_agree_bitwise(dtype):
    from oracle import gpt_stage_oracle as orc
    from parity_util import TOL, max_norm_err
    C, M = 3, 4
    shape = synth.StageShape(name="dpp", n_layers=3, hidden=128, n_heads=2, head_dim=64, ffn=256, seq=128,
                             batch=1, dtype=dtype, n_microbatches=M, bias_std=0.02, ln_jitter=0.1)
    print(f"[case] dpp driver {dtype} C={C} M={M}", flush=True)
    params_np = [{k: synth.to_storage(v, dtype) for k, v in synth.make_layer_params(shape, l, 0).items()}
                 for l in range(shape.n_layers)]
    runs = {}
    for name, cap in (("dfc", 0), ("bfc", 0), ("bfc_best_effort", 2 * C)):
        runs[name] = _run_dpp(shape, C, M, POLICY[name], cap, params_np)
    # memory behaviour as planned
    assert runs["dfc"][4].peak_live_stash == C and runs["bfc"][4].peak_live_stash == C * M
    assert runs["bfc_best_effort"][4].peak_live_stash == 2 * C
    # identical bits whatever the traversal
    for name in ("bfc", "bfc_best_effort"):
        for a, b in zip(runs["dfc"][:3], runs[name][:3]):
            for ta, tb in zip(a, b):
                assert np.array_equal(ta, tb), name
    # and the oracle of the whole stack
    p64 = [{k: v.astype(np.float64) for k, v in lp.items()} for lp in params_np]
    grads = None
    tol = TOL[dtype]
    ys, dxs, dps, cfg, _ = runs["dfc"]
    for m in range(M):
        x = synth.to_storage(synth.make_x(shape, 0, m), dtype).astype(np.float64)
        dy = synth.to_storage(synth.make_dy(shape, 0, m), dtype).astype(np.float64)
        y, dx, grads = orc.stage_fwd_bwd(x, dy, p64, shape.n_heads, shape.head_dim, shape.ln_eps, shape.gelu, grads=grads)
        assert max_norm_err(ys[m], y) <= tol and max_norm_err(dxs[m], dx) <= tol
    Lc = shape.n_layers // C
    for j in range(C):
        for l in range(Lc):
            for tid, name in enumerate(synth.TENSOR_NAMES):
                off, n = B.gpt_stage_param_offset(cfg, l, tid)
                ref = grads[j * Lc + l][name].reshape(-1)
                assert max_norm_err(dps[j][off:off + n], ref) <= tol, (j, l, name)


@pytest.mark.gpu
def test_dpp_driver_refuses_small_pools():
    import torch
    shape = synth.StageShape(name="dpp", n_layers=1, hidden=128, n_heads=2, head_dim=64, ffn=256, seq=64,
                             batch=1, dtype="fp32", n_microbatches=2)
    cfg = B.make_cfg(shape)
    n = B.gpt_stage_param_count(cfg)
    w = torch.zeros(n, device="cuda")
    ws = torch.empty(max(B.gpt_stage_workspace_bytes(cfg, 1), 256), dtype=torch.uint8, device="cuda")
    chunks = [B.gpt_stage_params(cfg=cfg, weights=w.data_ptr(), workspace=ws.data_ptr(), prepared=None, trace=None)] * 2
    t = [torch.zeros(1, 64, 128, device="cuda") for _ in range(2)]
    dps = [torch.zeros(n, device="cuda") for _ in range(2)]
    slot = B.gpt_dpp_stash_slot_bytes(chunks)
    stash = torch.empty(slot * 3, dtype=torch.uint8, device="cuda")     # breadth first needs 4
    act = torch.empty(B.gpt_dpp_act_slot_bytes(cfg) * 4, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.GptStageError) as e:
        B.gpt_dpp_run(B.GPT_DPP_BFC, chunks, t, t, [torch.empty_like(a) for a in t], [torch.empty_like(a) for a in t], dps, stash, act)
    assert e.value.code == B.GPTS_ENOMEM
    B.gpt_dpp_run(B.GPT_DPP_DFC, chunks, t, t, [torch.empty_like(a) for a in t], [torch.empty_like(a) for a in t], dps, stash, act)
    torch.cuda.synchronize()


@pytest.mark.gpu
def test_best_effort_allowance_from_the_memory_at_hand():
    """Without a caller-given allowance the best-effort policy runs as wide as the stash pool
    it is given allows, and gpt_dpp_allowance_from_free_memory sizes that pool from the
    device's free memory.  Results do not depend on the width."""
    import torch
    C, M = 2, 4
    shape = synth.StageShape(name="dpp_mem", n_layers=2, hidden=128, n_heads=2, head_dim=64, ffn=256, seq=128,
                             batch=1, dtype="bf16", n_microbatches=M, bias_std=0.02)
    params_np = [{k: synth.to_storage(v, "bf16") for k, v in synth.make_layer_params(shape, l, 0).items()}
                 for l in range(shape.n_layers)]
    ref = _run_dpp(shape, C, M, B.GPT_DPP_DFC, 0, params_np)
    cfg, chunks_probe = ref[3], None
    w = torch.zeros(B.gpt_stage_param_count(cfg), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(B.gpt_stage_workspace_bytes(cfg, 1), 256), dtype=torch.uint8, device="cuda")
    chunks_probe = [B.gpt_stage_params(cfg=cfg, weights=w.data_ptr(), workspace=ws.data_ptr(), prepared=None, trace=None)] * C
    slot = B.gpt_dpp_stash_slot_bytes(chunks_probe)
    free_b, _ = torch.cuda.mem_get_info()
    # plenty of memory: everything fits, i.e. plain breadth first
    n, sp, ap = B.gpt_dpp_allowance_from_free_memory(chunks_probe, M, 0)
    assert n == C * M and sp == n * slot and ap == (M + 1) * B.gpt_dpp_act_slot_bytes(cfg)
    # a reserve that leaves room for 5 slots: rounded down to whole windows of C = 2 chunks -> 4
    n, sp, ap = B.gpt_dpp_allowance_from_free_memory(chunks_probe, M, free_b - ap - 5 * slot - slot // 2)
    assert n == 4 and sp == 4 * slot
    n0, _, _ = B.gpt_dpp_allowance_from_free_memory(chunks_probe, M, free_b)
    assert n0 == 0
    # the driver with max_live_stash = 0 takes the width from the pool it is given
    for slots, want_peak in ((4, 4), (5, 4), (C * M, C * M), (3, 2)):
        got = _run_dpp(shape, C, M, B.GPT_DPP_BFC_BEST_EFFORT, 0, params_np, pool_slots=slots, expect_peak=want_peak)
        for a, b in zip(ref[:3], got[:3]):
            for ta, tb in zip(a, b):
                assert np.array_equal(ta, tb), slots


@pytest.mark.gpu
def test_dpp_full_size_four_chunks_against_the_stage_run():
    """The decoupled workload as 4 chunks of one layer x 8 micro-batches, breadth first and depth
    first: identical bits for both traversals, and the same numbers as the 4-layer stage run up
    to the rounding of the chunk-boundary activations (a chunk hands on bf16, the stage keeps
    its residual stream in fp32 between layers).  The stage run itself is tied to the oracle by
    the workload's own parity test; the forward output of micro-batch 0 is checked against the
    oracle here as well."""
    import torch
    from parity_util import gpu_run, max_norm_err
    shape = synth.WORKLOADS[3]
    C, M = 4, shape.n_microbatches
    print(f"[case] dpp full size {shape}", flush=True)
    params_np = synth.make_params(shape, 0)
    bfc = _run_dpp(shape, C, M, B.GPT_DPP_BFC, 0, params_np)
    print("[step] breadth first done", flush=True)
    dfc = _run_dpp(shape, C, M, B.GPT_DPP_DFC, 0, params_np)
    for a, b in zip(bfc[:3], dfc[:3]):
        for ta, tb in zip(a, b):
            assert np.array_equal(ta, tb)
    del dfc
    torch.cuda.empty_cache()
    print("[step] depth first == breadth first; running the 4-layer stage", flush=True)
    xs = [synth.make_x(shape, 0, m) for m in range(M)]
    dys = [synth.make_dy(shape, 0, m) for m in range(M)]
    ys, dxs, grads = gpu_run(shape, params_np, xs, dys, decoupled=True)
    cfg = bfc[3]
    worst = 0.0
    for m in range(M):
        worst = max(worst, max_norm_err(bfc[0][m], ys[m]), max_norm_err(bfc[1][m], dxs[m]))
    for j in range(C):
        for tid, name in enumerate(synth.TENSOR_NAMES):
            off, n = B.gpt_stage_param_offset(cfg, 0, tid)
            worst = max(worst, max_norm_err(bfc[2][j][off:off + n], grads[j][name].reshape(-1)))
    print(f"[parity] dpp 4 chunks vs stage: worst tensor-max-normalised difference {worst:.3e}", flush=True)
    # both are bf16 pipelines within 2e-2 of the exact result, rounded at different places
    # (measured 1.8e-2 apart at worst); an indexing or ordering mistake would be O(1)
    assert worst <= 3e-2
    # and the forward output of micro-batch 0 against the oracle itself
    from oracle import gpt_stage_oracle as orc
    from parity_util import TOL, p64
    y_ref, _ = orc.stage_fwd(xs[0].astype(np.float64), p64(params_np), shape.n_heads, shape.head_dim,
                             shape.ln_eps, shape.gelu)
    err = max_norm_err(bfc[0][0], y_ref)
    print(f"[parity] dpp 4 chunks, y of micro-batch 0 vs oracle: {err:.3e}", flush=True)
    assert err <= TOL["bf16"]


# ---- run-time scheduling: the ready set (host) ------------------------------------------------
def _lib_ready(policy, C, M, cap, x_at, dy_at, dynamic):
    order, steps, idle = B.gpt_dpp_simulate_ready(POLICY[policy], C, M, cap, x_at, dy_at, dynamic)
    return [("F" if p == B.GPT_DPP_FWD else "B", i, j) for p, i, j in order], steps, idle


@pytest.mark.parametrize("policy,cap", [("dfc", 0), ("bfc", 0), ("bfc_best_effort", 6)])
def test_ready_set_with_everything_present_is_the_static_plan(policy, cap):
    C, M = 3, 4
    want = dpo.traversal(policy, C, M, cap)
    for dynamic in (False, True):
        got, steps, idle = _lib_ready(policy, C, M, cap, None, None, dynamic)
        assert got == want and steps == len(want) and idle == 0
        assert dpo.ready_set_schedule(policy, C, M, cap, dynamic=dynamic) == (want, len(want), 0)


def test_ready_set_works_around_a_late_input_where_the_static_plan_idles():
    """Micro-batch 0's input is late.  The static breadth-first plan starts with F(0,0) and idles
    until it arrives; the ready-set scheduler runs the other micro-batches meanwhile."""
    C, M = 2, 4
    x_at = [6, 0, 0, 0]
    static = _lib_ready("bfc", C, M, 0, x_at, None, False)
    dynamic = _lib_ready("bfc", C, M, 0, x_at, None, True)
    assert static[2] == 6 and static[1] == 2 * C * M + 6          # six idle steps up front
    assert dynamic[2] == 0 and dynamic[1] == 2 * C * M            # none: six other tasks were ready
    assert dynamic[0][:6] == [("F", 1, 0), ("F", 2, 0), ("F", 3, 0), ("F", 1, 1), ("F", 2, 1), ("F", 3, 1)]
    assert dpo.dependencies_hold(dynamic[0], C, M)
    # backward on each chunk still in ascending micro-batch order
    for j in range(C):
        assert [i for ph, i, jj in dynamic[0] if ph == "B" and jj == j] == list(range(M))
    assert static == dpo.ready_set_schedule("bfc", C, M, 0, x_at, None, False)
    assert dynamic == dpo.ready_set_schedule("bfc", C, M, 0, x_at, None, True)


def test_ready_set_matches_the_oracle_on_random_arrivals_and_respects_memory():
    rng = np.random.default_rng(7)
    for trial in range(60):
        C, M = int(rng.integers(1, 5)), int(rng.integers(1, 7))
        policy = ("dfc", "bfc", "bfc_best_effort")[trial % 3]
        cap = int(rng.integers(0, C * M + 1)) if policy == "bfc_best_effort" else 0
        x_at = [int(v) for v in rng.integers(0, 3 * C * M, M)]
        dy_at = [int(v) for v in rng.integers(0, 5 * C * M, M)]
        for dynamic in (False, True):
            got = _lib_ready(policy, C, M, cap, x_at, dy_at, dynamic)
            want = dpo.ready_set_schedule(policy, C, M, cap, x_at, dy_at, dynamic)
            assert got == want, (policy, C, M, cap, x_at, dy_at, dynamic)
            order = got[0]
            assert dpo.dependencies_hold(order, C, M)
            assert dpo.peak_live_stash(order) <= dpo.peak_live_stash(dpo.traversal(policy, C, M, cap))
            assert len(order) == 2 * C * M
        # the ready set never needs more steps than the static plan
        assert _lib_ready(policy, C, M, cap, x_at, dy_at, True)[1] <= _lib_ready(policy, C, M, cap, x_at, dy_at, False)[1]


def test_ready_set_bad_arguments():
    with pytest.raises(B.GptStageError):
        B.gpt_dpp_simulate_ready(9, 2, 2)
    with pytest.raises(B.GptStageError):
        B.gpt_dpp_simulate_ready(B.GPT_DPP_BFC, 2, 2, x_at=[-1, 0])
    arr = (B.gpt_dpp_task * 2)()
    assert B.lib().gpt_dpp_simulate_ready(B.GPT_DPP_BFC, 2, 2, 0, None, None, 1, arr, 2, None, None) == B.GPTS_ENOMEM


@pytest.mark.gpu
def test_ready_set_driver_on_the_gpu_inputs_arriving_out_of_order():
    """gpt_dpp_run_ready with the inputs' arrival signalled by events: micro-batch 0's x is held
    back behind a spin kernel on a side stream, so the driver starts with the others; every
    result bit equals the static run, and an event that is never recorded ends in a time-out
    error, not a hang."""
    import torch
    C, M = 2, 3
    shape = synth.StageShape(name="dpp_ready", n_layers=2, hidden=128, n_heads=2, head_dim=64, ffn=256, seq=128,
                             batch=1, dtype="bf16", n_microbatches=M, bias_std=0.02)
    params_np = [{k: synth.to_storage(v, "bf16") for k, v in synth.make_layer_params(shape, l, 0).items()}
                 for l in range(shape.n_layers)]
    ref = _run_dpp(shape, C, M, B.GPT_DPP_BFC, 0, params_np)
    cfg = ref[3]
    nparam = B.gpt_stage_param_count(cfg)
    ws = torch.empty(max(B.gpt_stage_workspace_bytes(cfg, 1), 256), dtype=torch.uint8, device="cuda")
    chunks, weights, dps = [], [], []
    for j in range(C):
        w = torch.empty(nparam, dtype=torch.bfloat16, device="cuda")
        for tid, name in enumerate(synth.TENSOR_NAMES):
            off, n = B.gpt_stage_param_offset(cfg, 0, tid)
            w[off:off + n].copy_(B.to_device(params_np[j][name].reshape(-1), "bf16"))
        weights.append(w)
        dps.append(torch.zeros(nparam, dtype=torch.float32, device="cuda"))
        chunks.append(B.gpt_stage_params(cfg=cfg, weights=w.data_ptr(), workspace=ws.data_ptr(), prepared=None, trace=None))
    xs = [B.to_device(synth.make_x(shape, 0, m), "bf16") for m in range(M)]
    dys = [B.to_device(synth.make_dy(shape, 0, m), "bf16") for m in range(M)]
    ys, dxs = [torch.empty_like(x) for x in xs], [torch.empty_like(x) for x in xs]
    stash = torch.empty(B.gpt_dpp_stash_slot_bytes(chunks) * C * M, dtype=torch.uint8, device="cuda")
    act = torch.empty(B.gpt_dpp_act_slot_bytes(cfg) * (M + 1), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    x_ready = [torch.cuda.Event() for _ in range(M)]
    torch.cuda.synchronize()
    x_ready[1].record()
    x_ready[2].record()                       # present at once
    with torch.cuda.stream(side):
        torch.cuda._sleep(200_000_000)        # ~0.1 s before micro-batch 0's input "arrives"
        x_ready[0].record(side)
    rep, order = B.gpt_dpp_run_ready(B.GPT_DPP_BFC, chunks, xs, dys, ys, dxs, dps, stash, act, x_ready=x_ready)
    torch.cuda.synchronize()
    assert rep.n_tasks == 2 * C * M
    assert order[0] == (B.GPT_DPP_FWD, 1, 0)                      # did not wait for micro-batch 0
    named = [("F" if p == B.GPT_DPP_FWD else "B", i, j) for p, i, j in order]
    assert dpo.dependencies_hold(named, C, M)
    got = ([B.to_host(t) for t in ys], [B.to_host(t) for t in dxs], [t.cpu().numpy() for t in dps])
    for a, b in zip(ref[:3], got):
        for ta, tb in zip(a, b):
            assert np.array_equal(ta, tb)
    # an input that never arrives: the call gives up instead of waiting for ever
    never = torch.cuda.Event()
    never.record(side)                        # creates the event handle ...
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        torch.cuda._sleep(2_000_000_000)      # ... and this re-record completes only after ~1 s
        never.record(side)
    for d in dps:
        d.zero_()
    with pytest.raises(B.GptStageError) as e:
        B.gpt_dpp_run_ready(B.GPT_DPP_BFC, chunks, xs, dys, ys, dxs, dps, stash, act,
                            dy_ready=[never, None, None], timeout_seconds=0.2)
    assert e.value.code == B.GPTS_EHIP and "did not arrive" in str(e.value)
    torch.cuda.synchronize()


@pytest.mark.gpu
def test_dpp_weight_phase_per_chunk_and_window():
    """With a gradient-stash pool the driver runs data-phase backward tasks and one weight phase
    per chunk and window.  Same y, dx, bias and LayerNorm gradients bit for bit; weight gradients
    bit-identical where the weight phase takes one product per micro-batch (depth first: windows
    of one) and equal up to the fp32 summation order where it contracts over a window in one
    launch (breadth first, >= 100 tiles of 256x256)."""
    from parity_util import max_norm_err
    C, M = 2, 3
    shape = synth.StageShape(name="dpp_wp", n_layers=2, hidden=2048, n_heads=16, head_dim=128, ffn=4096, seq=256,
                             batch=1, dtype="bf16", n_microbatches=M, bias_std=0.02, ln_jitter=0.1)
    params_np = [{k: synth.to_storage(v, "bf16") for k, v in synth.make_layer_params(shape, l, 0).items()}
                 for l in range(shape.n_layers)]
    ref = _run_dpp(shape, C, M, B.GPT_DPP_BFC, 0, params_np)
    cfg = ref[3]
    weights = {}
    for tid, name in enumerate(synth.TENSOR_NAMES):
        weights[name] = B.gpt_stage_param_offset(cfg, 0, tid)
    for policy, cap, one_launch in ((B.GPT_DPP_DFC, 0, False), (B.GPT_DPP_BFC, 0, True),
                                    (B.GPT_DPP_BFC_BEST_EFFORT, 2 * C, True)):
        got = _run_dpp(shape, C, M, policy, cap, params_np, weight_phase=True)
        for a, b in zip(ref[0] + ref[1], got[0] + got[1]):
            assert np.array_equal(a, b)
        changed = 0
        for j in range(C):
            for name, (off, n) in weights.items():
                a, b = ref[2][j][off:off + n], got[2][j][off:off + n]
                if name in ("w_qkv", "w_fc1", "w_fc2") and one_launch:
                    assert max_norm_err(b, a) < 2e-6, (policy, j, name)
                    changed += int(not np.array_equal(a, b))
                else:
                    assert np.array_equal(a, b), (policy, j, name)
        assert (changed > 0) == one_launch
    # pools too small for the fixed slot pattern are refused before anything runs
    import torch
    chunks = [B.gpt_stage_params(cfg=cfg, weights=0x10000, workspace=0x20000, prepared=None, trace=None)] * C
    t = [torch.zeros(1, 256, 2048, dtype=torch.bfloat16, device="cuda") for _ in range(M)]
    dps = [torch.zeros(8, device="cuda") for _ in range(C)]
    stash = torch.empty(B.gpt_dpp_stash_slot_bytes(chunks) * (C * M - 1), dtype=torch.uint8, device="cuda")
    act = torch.empty(B.gpt_dpp_act_slot_bytes(cfg) * 8, dtype=torch.uint8, device="cuda")
    gp = torch.empty(B.gpt_dpp_grad_slot_bytes(chunks) * M, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.GptStageError) as e:
        B.gpt_dpp_run(B.GPT_DPP_BFC, chunks, t, t, t, t, dps, stash, act, grad_pool=gp)
    assert e.value.code == B.GPTS_ENOMEM
