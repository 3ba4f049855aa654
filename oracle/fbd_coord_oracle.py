"""The communication coordinator's rule, stated plainly -- TEST INFRASTRUCTURE ONLY.

Section 4.2 (MegaFBD, "communication coordinator"): "start a collective only after confirming
that all ranks in the group have issued the same request"; ready collectives are executed
"in ascending group order".  This module states that rule with Python sets and lists -- no
bit vectors, no tables -- so that the library's bit-vector implementation can be compared
with it.  It also models what the section warns about: control threads that start requests
without verification.

A program is, per virtual rank, the list of groups it performs collectives in, in order; a
rank posts its next request only when its previous collective is done.
"""
from __future__ import annotations


def expected_mask(group, n_ranks: int) -> str:
    """One character per virtual rank, rank 0 leftmost: '1' for the group's members."""
    return "".join("1" if r in set(group) else "0" for r in range(n_ranks))


def run_with_coordinator(groups, programs):
    """groups: list of member lists; programs: list (per rank) of group indices.
    Returns (log, deadlocked): the collectives in execution order."""
    pc = [0] * len(programs)
    posted = {}                       # rank -> group it is waiting in
    log = []
    while True:
        for r, prog in enumerate(programs):
            if r not in posted and pc[r] < len(prog):
                posted[r] = prog[pc[r]]
        if not posted:
            return log, False
        ready = [g for g, members in enumerate(groups)
                 if all(posted.get(r) == g for r in members)]      # all members, same request
        if not ready:
            return log, True
        for g in sorted(ready):                                      # ascending group order
            log.append(g)
            for r in groups[g]:
                del posted[r]
                pc[r] += 1


def run_without_verification(groups, programs, control_of):
    """Every control thread starts the oldest request it holds and is busy with it until the
    collective completes (every member's request for the group started by its own thread)."""
    n_control = max(control_of) + 1
    pc = [0] * len(programs)
    queue = [[] for _ in range(n_control)]
    busy = [None] * n_control
    posted = set()
    log = []
    while True:
        progress = False
        for r, prog in enumerate(programs):
            if r not in posted and pc[r] < len(prog):
                queue[control_of[r]].append(r)
                posted.add(r)
                progress = True
        for k in range(n_control):
            if busy[k] is None and queue[k]:
                busy[k] = queue[k].pop(0)
                progress = True
        for g, members in enumerate(groups):
            if all(busy[control_of[r]] == r and programs[r][pc[r]] == g for r in members):
                log.append(g)
                for r in members:
                    busy[control_of[r]] = None
                    pc[r] += 1
                    posted.discard(r)
                progress = True
        if all(pc[r] >= len(p) for r, p in enumerate(programs)):
            return log, False
        if not progress:
            return log, True
