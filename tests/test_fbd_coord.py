"""Communication coordinator (section 4.2, MegaFBD), simulated on the host -- no GPU.

The oracle states the section's rule with sets ("start a collective only after ... all ranks in
the group have issued the same request", "ascending group order"); the library implements the
section's four steps with bit-vector tables.  Pins: the printed example (eight threads, group
{0,1,2,3} expects 11110000), the Rank 0 / 1 / 2 scenario of the section (deadlock without
verification, none with the coordinator), and invariants on random programs."""
import os

import numpy as np
import pytest

from oracle import fbd_coord_oracle as fco
from paper_2507_19845_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "coordinator_mask.txt")


def _golden():
    kv = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            kv[k] = v
    return int(kv["threads"][0]), [int(x) for x in kv["group"]], kv["expected"][0]


def test_printed_example_mask():
    n, group, expected = _golden()
    assert fco.expected_mask(group, n) == expected == "11110000"
    h = B.gpt_fbd_coord_create(n, [group, [4, 5, 6, 7]], [0, 0, 0, 0, 1, 1, 1, 1])
    try:
        assert B.gpt_fbd_coord_expected(h, 0, n) == expected
        assert B.gpt_fbd_coord_expected(h, 1, n) == "00001111"
    finally:
        B.gpt_fbd_coord_destroy(h)


# the section's scenario: rank 0 wants to talk to rank 2, rank 2 to rank 1; ranks 0 and 1
# share a control thread
SCENARIO_GROUPS = [[0, 2], [1, 2]]
SCENARIO_PROGRAMS = [[0], [1], [1, 0]]
SCENARIO_CONTROL = [0, 0, 1]


def test_scenario_oracle():
    log, dead = fco.run_without_verification(SCENARIO_GROUPS, SCENARIO_PROGRAMS, SCENARIO_CONTROL)
    assert dead and log == []                      # 0-2 started first, 1-2 blocked behind it
    log, dead = fco.run_with_coordinator(SCENARIO_GROUPS, SCENARIO_PROGRAMS)
    assert not dead and log == [1, 0]              # 1-2 is the one everybody asked for; then 0-2


def test_scenario_library_step_by_step():
    h = B.gpt_fbd_coord_create(3, SCENARIO_GROUPS, SCENARIO_CONTROL)
    try:
        B.gpt_fbd_coord_register(h, 0, 0)          # rank 0 -> group {0,2}
        B.gpt_fbd_coord_register(h, 1, 1)          # rank 1 -> group {1,2}
        B.gpt_fbd_coord_register(h, 2, 1)          # rank 2 -> group {1,2}
        # before alignment no control thread sees a complete vector
        assert B.gpt_fbd_coord_ready(h, 0, 2) == [] and B.gpt_fbd_coord_ready(h, 1, 2) == []
        B.gpt_fbd_coord_align(h)
        assert B.gpt_fbd_coord_ready(h, 0, 2) == [1] == B.gpt_fbd_coord_ready(h, 1, 2)
        assert B.gpt_fbd_coord_execute(h, 2) == [1]
        assert B.gpt_fbd_coord_ready(h, 0, 2) == []   # group 0 still waits for rank 2
        B.gpt_fbd_coord_register(h, 2, 0)
        B.gpt_fbd_coord_align(h)
        assert B.gpt_fbd_coord_execute(h, 2) == [0]
        with pytest.raises(B.GptStageError):
            B.gpt_fbd_coord_register(h, 1, 0)         # rank 1 is not in group {0,2}
    finally:
        B.gpt_fbd_coord_destroy(h)


def test_scenario_library_simulation():
    h = B.gpt_fbd_coord_create(3, SCENARIO_GROUPS, SCENARIO_CONTROL)
    try:
        assert B.gpt_fbd_coord_simulate(h, SCENARIO_PROGRAMS, verify=False) == ([], True)
        assert B.gpt_fbd_coord_simulate(h, SCENARIO_PROGRAMS, verify=True) == ([1, 0], False)
    finally:
        B.gpt_fbd_coord_destroy(h)


def _random_case(rng, n_ranks, n_groups, n_coll, n_control):
    groups = []
    while len(groups) < n_groups:
        k = int(rng.integers(2, min(5, n_ranks) + 1))
        g = sorted(rng.choice(n_ranks, size=k, replace=False).tolist())
        if g not in groups:
            groups.append(g)
    # consistent programs: a global sequence of collectives, each rank sees its own in order
    seq = rng.integers(0, n_groups, size=n_coll).tolist()
    programs = [[g for g in seq if r in groups[g]] for r in range(n_ranks)]
    control = sorted(rng.integers(0, n_control, size=n_ranks).tolist())
    control = [c if c < max(control) + 1 else 0 for c in control]
    # make control thread ids dense
    ids = {c: i for i, c in enumerate(sorted(set(control)))}
    return groups, programs, [ids[c] for c in control], seq


@pytest.mark.parametrize("seed", range(12))
def test_random_consistent_programs_never_deadlock_and_match_oracle(seed):
    rng = np.random.default_rng(seed)
    n_ranks = int(rng.integers(3, 70 if seed % 3 == 0 else 12))    # also more than 64 ranks: two words per vector
    groups, programs, control, seq = _random_case(rng, n_ranks, int(rng.integers(2, 9)), int(rng.integers(1, 40)),
                                                  int(rng.integers(1, 5)))
    ref_log, ref_dead = fco.run_with_coordinator(groups, programs)
    assert not ref_dead and sorted(ref_log) == sorted(seq)        # every collective, exactly once
    # each rank's collectives happen in its program order
    for r, prog in enumerate(programs):
        assert [g for g in ref_log if r in groups[g]] == prog
    h = B.gpt_fbd_coord_create(n_ranks, groups, control)
    try:
        assert B.gpt_fbd_coord_simulate(h, programs, verify=True) == (ref_log, False)
        naive = B.gpt_fbd_coord_simulate(h, programs, verify=False)
        assert naive == fco.run_without_verification(groups, programs, control)
    finally:
        B.gpt_fbd_coord_destroy(h)


def test_inconsistent_programs_are_reported_not_hung():
    groups = [[0, 1], [1, 2], [0, 2]]
    programs = [[0], [1], [2]]          # a cycle: nobody's request is ever matched
    assert fco.run_with_coordinator(groups, programs) == ([], True)
    h = B.gpt_fbd_coord_create(3, groups, [0, 1, 2])
    try:
        assert B.gpt_fbd_coord_simulate(h, programs, verify=True) == ([], True)
    finally:
        B.gpt_fbd_coord_destroy(h)


def test_ascending_group_order_within_a_round():
    groups = [[4, 5], [2, 3], [0, 1]]
    programs = [[2], [2], [1], [1], [0], [0]]
    log, dead = fco.run_with_coordinator(groups, programs)
    assert (log, dead) == ([0, 1, 2], False)
    h = B.gpt_fbd_coord_create(6, groups, [0, 0, 1, 1, 2, 2])
    try:
        assert B.gpt_fbd_coord_simulate(h, programs, verify=True) == ([0, 1, 2], False)
    finally:
        B.gpt_fbd_coord_destroy(h)
