"""Traversal orders of the (micro-batch, model chunk) task matrix -- TEST INFRASTRUCTURE ONLY.

Plain Python statement of the schedules of section 5.2 (MegaDPP, "parallel scheduler"):
the compute tasks of one iteration form a matrix indexed by (model chunk, micro-batch), task
"i-j" processes micro-batch i on chunk j (figure 3 caption), and a schedule is a traversal
order of that matrix.  Only tests, the smoke check and the CPU leg of the benchmark may import
this module; the library never does.

A task is a tuple (phase, i, j) with phase "F" (forward) or "B" (backward).  Chunks sit one
after the other: F(i,j) needs F(i,j-1); B(i,j) needs F(i,j) and B(i,j+1).

Readings where the section is silent:
  * depth first, all chunks on one device: the backward of a micro-batch follows its forward
    immediately ("lets the corresponding backward pass start earlier, releases activation
    memory sooner");
  * breadth first: every micro-batch on chunk 0, then on chunk 1, ...; backward likewise from
    the last chunk down, so that a chunk's gradients are complete as soon as possible;
  * best effort ("as long as it does not cause" out-of-memory): breadth first over windows of
    W consecutive micro-batches, W the largest count whose activation stashes (one per task in
    flight, n_chunks per micro-batch) fit the given allowance, never fewer than one.
"""
from __future__ import annotations


def task_name(i: int, j: int) -> str:
    """Figure 3 caption: "i-j" = micro-batch i on chunk j."""
    return f"{i}-{j}"


def task_matrix(n_chunks: int, n_microbatches: int):
    """The matrix of forward tasks, rows = micro-batches, columns = chunks."""
    return [[task_name(i, j) for j in range(n_chunks)] for i in range(n_microbatches)]


def depth_first(n_chunks: int, n_microbatches: int):
    order = []
    for i in range(n_microbatches):              # same micro-batch across different chunks first
        for j in range(n_chunks):
            order.append(("F", i, j))
        for j in reversed(range(n_chunks)):
            order.append(("B", i, j))
    return order


def breadth_first(n_chunks: int, n_microbatches: int):
    order = []
    for j in range(n_chunks):                    # different micro-batches on the same chunk first
        for i in range(n_microbatches):
            order.append(("F", i, j))
    for j in reversed(range(n_chunks)):
        for i in range(n_microbatches):
            order.append(("B", i, j))
    return order


def best_effort_breadth_first(n_chunks: int, n_microbatches: int, max_live_stash: int):
    per_microbatch = n_chunks                    # stashes a micro-batch holds at its peak
    w = max(1, min(n_microbatches, max_live_stash // per_microbatch))
    order = []
    for start in range(0, n_microbatches, w):
        group = range(start, min(n_microbatches, start + w))
        for j in range(n_chunks):
            for i in group:
                order.append(("F", i, j))
        for j in reversed(range(n_chunks)):
            for i in group:
                order.append(("B", i, j))
    return order


def traversal(policy: str, n_chunks: int, n_microbatches: int, max_live_stash: int = 0):
    if policy == "dfc":
        return depth_first(n_chunks, n_microbatches)
    if policy == "bfc":
        return breadth_first(n_chunks, n_microbatches)
    if policy == "bfc_best_effort":
        return best_effort_breadth_first(n_chunks, n_microbatches, max_live_stash)
    raise ValueError(policy)


def peak_live_stash(order) -> int:
    """Largest number of activation stashes alive at once: one is created by every forward
    task and released by the matching backward task."""
    live = peak = 0
    for phase, _, _ in order:
        live += 1 if phase == "F" else -1
        peak = max(peak, live)
    return peak


def dependencies_hold(order, n_chunks: int, n_microbatches: int) -> bool:
    """Every task exactly once, each after the tasks it needs."""
    done = set()
    for t in order:
        phase, i, j = t
        if t in done or not (0 <= i < n_microbatches and 0 <= j < n_chunks):
            return False
        if phase == "F":
            if j > 0 and ("F", i, j - 1) not in done:
                return False
        else:
            if ("F", i, j) not in done:
                return False
            if j < n_chunks - 1 and ("B", i, j + 1) not in done:
                return False
        done.add(t)
    return len(done) == 2 * n_chunks * n_microbatches


def gradient_ready_position(order, n_chunks: int):
    """Index in the order of the last backward task of each chunk: from there on the chunk's
    gradients are complete and could be exchanged."""
    last = [None] * n_chunks
    for pos, (phase, _, j) in enumerate(order):
        if phase == "B":
            last[j] = pos
    return last


# ---- run-time scheduling: the ready set -----------------------------------------------------
def ready_set_schedule(policy: str, n_chunks: int, n_microbatches: int, max_live_stash: int = 0,
                       x_at=None, dy_at=None, dynamic: bool = True):
    """Section 5.2, lightweight communication library: "a compute thread can always pick the
    highest-priority ready input for execution".  Discrete time, one task per step.

    External inputs: x of micro-batch i is present from step x_at[i] (needed by F(i,0)), dy of
    micro-batch i from step dy_at[i] (needed by B(i,C-1)); None = present from step 0.
    A task may run at a step if
      * the tasks it needs (see dependencies_hold) have run and its external input is present;
      * backward tasks of one chunk run in ascending micro-batch order (gradient accumulation
        order is that of the static plan);
      * memory: a forward task needs a free stash slot; F(i,0) additionally needs that the free
        slots, minus what the micro-batches in flight still need to reach the last chunk, cover
        all n_chunks of the new micro-batch -- and n_chunks more when a lower-numbered micro-batch
        has not started yet (its backward tasks go first, so it must be able to pass through).
        The number of slots is the peak of the static plan.
    Priority = position in the static plan of `policy`.  dynamic=False: only the plan's next
    task is considered (a static schedule waiting for its input).
    Returns (order, n_steps, idle_steps)."""
    C, M = n_chunks, n_microbatches
    plan = traversal(policy, C, M, max_live_stash)
    slots = peak_live_stash(plan)
    x_at = [0] * M if x_at is None else list(x_at)
    dy_at = [0] * M if dy_at is None else list(dy_at)
    done, order = set(), []
    step = idle = 0

    def free_slots():
        return slots - sum(1 for (ph, i, j) in done if ph == "F") + sum(1 for (ph, i, j) in done if ph == "B")

    def still_needed():
        need = 0
        for i in range(M):
            fwd = sum(1 for j in range(C) if ("F", i, j) in done)
            if 0 < fwd < C:
                need += C - fwd
        return need

    def can_run(t):
        ph, i, j = t
        if ph == "F":
            if j == 0:
                if x_at[i] > step:
                    return False
                lower_started = all(("F", k, 0) in done for k in range(i))
                return free_slots() - still_needed() >= (C if lower_started else 2 * C)
            return ("F", i, j - 1) in done and free_slots() > 0
        if ("F", i, j) not in done:
            return False
        if any(("B", k, j) not in done for k in range(i)):
            return False
        if j == C - 1:
            return dy_at[i] <= step
        return ("B", i, j + 1) in done

    guard = max(x_at + dy_at) + 4 * len(plan) + 8
    while len(done) < len(plan):
        assert step <= guard, "no progress"
        pending = [t for t in plan if t not in done]
        candidates = pending if dynamic else pending[:1]
        pick = next((t for t in candidates if can_run(t)), None)
        if pick is None:
            idle += 1
        else:
            done.add(pick)
            order.append(pick)
        step += 1
    return order, step, idle
