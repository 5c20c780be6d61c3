"""The library's epoch schedule (host logic behind the C ABI, no GPU involved) against the
set-based oracle of the same passage (paper Section 3.2), step by step and bit for bit."""
import itertools

import numpy as np
import pytest

from oracle import schedule_oracle as so
from paper_2002_02885_amd import binding


def _native(n, batch):
    s = binding.Schedule(n, batch)
    out = []
    try:
        while True:
            r = s.next()
            if r is None:
                break
            out.append((list(map(int, r[0])), list(map(int, r[1])), r[2]))
        used = list(s.used())
        assert s.next() is None                      # stays at the end
    finally:
        s.destroy()
    return out, used


def _oracle(n, batch):
    return [(st["idx"], st["rows"], st["lead"]) for st in so.epoch_schedule(n, list(batch))]


def test_all_small_cases_agree_with_the_oracle():
    for n in (1, 2, 5, 7, 12, 64, 65, 130):
        for K in (1, 2, 3):
            for batch in itertools.product((1, 2, 3, 5, 8, 64), repeat=K):
                got, used = _native(n, list(batch))
                assert got == _oracle(n, batch), (n, batch)
                assert used == [n] * K


def test_paper_sized_cases_agree_with_the_oracle():
    got, _ = _native(10000, [20, 50, 100])           # the step-count example of Section 3.3
    assert got == _oracle(10000, [20, 50, 100]) and len(got) == 500
    rng = np.random.default_rng(3)
    for _ in range(5):
        K = int(rng.integers(1, 9))
        batch = [int(b) for b in rng.integers(1, 300, size=K)]
        n = int(rng.integers(1, 5000))
        got, used = _native(n, batch)
        assert got == _oracle(n, batch), (n, batch)
        assert used == [n] * K


def test_progress_is_reported_while_the_epoch_runs():
    s = binding.Schedule(1000, [100, 50, 80])
    try:
        for _ in range(10):
            s.next()
        assert list(s.used()) == [1000, 500, 800]    # Section 3.2: 50 % and 80 % when the first member is done
    finally:
        s.destroy()


def test_argument_errors():
    for n, batch in ((0, [4]), (10, []), (10, [4, 0]), (10, [1] * 257)):
        with pytest.raises(binding.PackError) as e:
            binding.Schedule(n, batch)
        assert e.value.status == binding.PACK_EINVAL
