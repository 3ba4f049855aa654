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
