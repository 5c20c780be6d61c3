"""Pins of the epoch-schedule oracle (paper Section 3.2 progress tracking, Section 3.3 step
counts): the numbers the paper prints, closed forms for batch sizes that divide the dataset, the
exactly-once property, and brute force over all small cases against a second formulation."""
import itertools
import os

import pytest

from oracle import schedule_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "schedule_worked_examples.txt")


def _gold():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def _member_steps(steps, k):
    return sum(1 for st in steps if st["rows"][k] > 0)


def test_progress_when_the_largest_batch_finishes_matches_the_papers_numbers():
    g = _gold()
    for n in (100, 1000, 4000):
        steps = so.epoch_schedule(n, [100, 50, 80])
        first_phase = n // 100
        assert all(st["lead"] == 0 for st in steps[:first_phase]) and steps[first_phase]["lead"] == 2
        prog = so.progress_after(steps, n, 3, first_phase)
        assert prog[0] == 1.0
        assert prog[1] == g["progress_batch50_when_batch100_done"]
        assert prog[2] == g["progress_batch80_when_batch100_done"]


def test_step_counts_match_the_papers_numbers():
    g = _gold()
    n = int(g["samples_sec33"])
    steps = so.epoch_schedule(n, [20, 50, 100])
    assert _member_steps(steps, 0) == g["steps_batch20"]
    assert _member_steps(steps, 1) == g["steps_batch50"]
    assert _member_steps(steps, 2) == g["steps_batch100"]
    # the batch-100 member is the one that leaves first, after its 100 steps
    assert all(st["rows"][2] == 100 for st in steps[:100]) and all(st["rows"][2] == 0 for st in steps[100:])
    # divisible case: the packed epoch is as long as the slowest member's own epoch
    assert len(steps) == n // 20


def _check_exactly_once(n, batch, steps):
    K = len(batch)
    seen = [[] for _ in range(K)]
    for st in steps:
        live = [k for k in range(K) if st["rows"][k] > 0]
        assert live, "a step must train somebody"
        assert len(st["idx"]) == max(st["rows"])
        assert len(st["idx"]) <= batch[st["lead"]] and st["rows"][st["lead"]] == len(st["idx"])
        for k in live:
            assert st["rows"][k] == min(batch[k], len(st["idx"]))
            seen[k].extend(st["idx"][:st["rows"][k]])
    for k in range(K):
        assert sorted(seen[k]) == list(range(n)), f"member {k} must see every sample exactly once"


def _phase_formulation(n, batch):
    """A second way to the same schedule, by position arithmetic instead of bookkeeping of used
    samples: every member takes leading rows, so of the samples a phase consumes a member with
    batch size b leaves over exactly those that stood at position >= b inside their shared batch;
    what the phase did not touch stays left over."""
    K = len(batch)
    order = sorted(range(K), key=lambda k: (-batch[k], k))
    left = [list(range(n)) for _ in range(K)]
    steps, done = [], set()
    for lead in order:
        if not left[lead]:               # finished together with an earlier leading member
            done.add(lead)
            continue
        pool = sorted(left[lead])
        shared_batches = [pool[s:s + batch[lead]] for s in range(0, len(pool), batch[lead])]
        for shared in shared_batches:
            rows = [0 if k in done else min(batch[k], len(shared)) for k in range(K)]
            steps.append({"idx": shared, "rows": rows, "lead": lead})
        in_pool = set(pool)
        for k in range(K):
            if k in done:
                continue
            untouched = [p for p in left[k] if p not in in_pool]
            left[k] = untouched + [p for shared in shared_batches for p in shared[batch[k]:]]
        done.add(lead)
    return steps


def test_brute_force_small_cases_against_position_arithmetic():
    for n in (1, 2, 5, 7, 12):
        for K in (1, 2, 3):
            for batch in itertools.product((1, 2, 3, 5, 8), repeat=K):
                steps = so.epoch_schedule(n, list(batch))
                _check_exactly_once(n, batch, steps)
                other = _phase_formulation(n, list(batch))
                assert [(s["idx"], s["rows"], s["lead"]) for s in steps] == \
                       [(s["idx"], s["rows"], s["lead"]) for s in other], (n, batch)


def test_ragged_and_oversized_batches():
    steps = so.epoch_schedule(10, [8, 5])
    assert [s["idx"] for s in steps] == [[0, 1, 2, 3, 4, 5, 6, 7], [8, 9], [5, 6, 7]]
    assert [s["rows"] for s in steps] == [[8, 5], [2, 2], [0, 3]]
    steps = so.epoch_schedule(3, [64])          # batch larger than the dataset: one short step
    assert [s["rows"] for s in steps] == [[3]]
    _check_exactly_once(1000, [128, 96, 33, 128], so.epoch_schedule(1000, [128, 96, 33, 128]))


def test_equal_batches_share_every_step():
    steps = so.epoch_schedule(40, [10, 10, 10])
    assert len(steps) == 4 and all(s["rows"] == [10, 10, 10] and s["lead"] == 0 for s in steps)


def test_a_planted_mistake_is_caught():
    """Taking the remainder of the WRONG member (any but the one with the largest batch) as the
    pool repeats samples: the exactly-once check must see it."""
    n, batch = 20, [10, 4, 6]
    steps = so.epoch_schedule(n, batch)
    bad = [dict(s, idx=list(s["idx"])) for s in steps]
    first_second_phase = n // 10
    bad[first_second_phase]["idx"][0] = 0       # a sample member 2 has already used
    with pytest.raises(AssertionError):
        _check_exactly_once(n, batch, bad)


def test_argument_errors():
    for args in ((0, [4]), (10, []), (10, [4, 0])):
        with pytest.raises(ValueError):
            so.epoch_schedule(*args)
