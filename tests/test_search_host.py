"""The library's search logic (host code behind the C ABI, no GPU involved) against the oracle of
the same passages (paper Section 5): integer results, compared exactly."""
import numpy as np
import pytest

import workloads as wl
from oracle import search_oracle as so
from paper_2002_02885_amd import binding

CAT = [1 if c else 0 for c in so.CATEGORICAL]


def test_distance_agrees_on_every_pair_of_a_sample_and_on_the_papers_example():
    confs = so.all_configurations()
    a, b = so.configuration(20, "sgd", 0.01, "relu"), so.configuration(40, "adagrad", 0.01, "relu")
    assert binding.config_distance(a, b, CAT) == so.distance(a, b) == 5
    rng = np.random.default_rng(0)
    pick = [confs[i] for i in rng.choice(len(confs), size=60, replace=False)]
    for x in pick:
        for y in pick:
            assert binding.config_distance(x, y, CAT) == so.distance(x, y)


def test_knn_grouping_agrees_with_the_oracle():
    confs_all = so.all_configurations()
    rng = np.random.default_rng(1)
    for trial in range(200):
        T = int(rng.integers(1, 60))
        confs = [confs_all[i] for i in rng.integers(0, len(confs_all), size=T)]
        need = [int(v) for v in rng.integers(1, 12, size=T)]
        capacity = int(rng.integers(3, 50))
        threshold = int(rng.integers(0, 14))
        draws = rng.random(T)
        want = [sorted(g) for g in so.pack_opt_knn(confs, need, capacity, threshold, draws)]
        assert binding.opt_knn(confs, CAT, need, capacity, threshold, draws) == want, (trial, T)
    # the hand-worked cases of the oracle's pins
    line = [(0, 1, 2, 3), (1, 1, 2, 3), (2, 1, 2, 3), (6, 1, 2, 3), (7, 1, 2, 3)]
    assert binding.opt_knn(line, CAT, [1] * 5, 3, 2, [0.5, 0.0, 0, 0, 0]) == [[0, 1, 2], [3, 4]]
    assert binding.opt_knn(line, CAT, [1, 5, 1, 1, 1], 3, 2, [0.5, 0.0, 0.0, 0, 0]) == [[0, 2], [1], [3, 4]]


def test_comparison_heuristics_agree_with_the_oracle():
    confs_all = so.all_configurations()
    rng = np.random.default_rng(2)
    for trial in range(100):
        T = int(rng.integers(1, 70))
        confs = [confs_all[i] for i in rng.integers(0, len(confs_all), size=T)]
        need = [int(v) for v in rng.integers(1, 9, size=T)]
        capacity = int(rng.integers(2, 30))
        want = so.pack_batchsize(confs, need, capacity)
        assert binding.opt_batchsize([c[0] for c in confs], need, capacity) == want
        m = int(rng.integers(1, 12))
        perm = [int(i) for i in rng.permutation(T)]
        assert binding.opt_random(T, m, perm) == [sorted(g) for g in so.pack_random(T, m, perm)]


def test_hyperband_plan_and_halving_agree_with_the_oracle():
    for R, eta in ((81, 3), (9, 3), (1, 3), (27, 3), (16, 2), (100, 3), (64, 4), (7, 2)):
        assert binding.hyperband_plan(R, eta) == so.hyperband_brackets(R, eta), (R, eta)
    rng = np.random.default_rng(3)
    for _ in range(100):
        n = int(rng.integers(1, 40))
        loss = np.round(rng.random(n), 1).astype(np.float32)          # many ties
        keep = int(rng.integers(0, n + 1))
        assert binding.halving_keep(loss, keep) == so.keep_best([float(v) for v in loss], keep)
    # diverged configurations (NaN, inf) never displace a finite loss: same rule on both sides
    for _ in range(200):
        n = int(rng.integers(1, 30))
        loss = np.round(rng.random(n), 1).astype(np.float32)
        loss[rng.random(n) < 0.3] = np.nan
        loss[rng.random(n) < 0.2] = np.inf
        keep = int(rng.integers(0, n + 1))
        got = binding.halving_keep(loss, keep)
        assert got == so.keep_best([float(v) for v in loss], keep)
        n_finite = int(np.isfinite(loss).sum())
        assert sum(bool(np.isfinite(loss[i])) for i in got) == min(keep, n_finite)
    assert binding.halving_keep(np.array([np.nan, 5.0, np.inf, 1.0], dtype=np.float32), 2) == [1, 3]


def test_argument_errors():
    with pytest.raises(binding.PackError):
        binding.opt_knn([(0, 0, 0, 0)], CAT, [1], 4, 2, [1.0])        # draw outside [0, 1)
    with pytest.raises(binding.PackError):
        binding.opt_random(3, 2, [0, 1, 1])
    with pytest.raises(binding.PackError):
        binding.opt_random(3, 0, [0, 1, 2])
    with pytest.raises(binding.PackError):
        binding.hyperband_plan(81, 1)
    with pytest.raises(binding.PackError):
        binding.halving_keep([1.0, 2.0], 3)


def test_memory_model_counts_parameters_state_and_activations():
    layers = wl.mlp([64, 32], 10)
    n = wl.num_params(layers, (1, 1, 96))
    sgd = binding.estimate_bytes(32, (1, 1, 96), "f32", layers, 32, "sgd")
    adam = binding.estimate_bytes(32, (1, 1, 96), "f32", layers, 32, "adam")
    mom = binding.estimate_bytes(32, (1, 1, 96), "f32", layers, 32, "momentum")
    assert sgd >= 8 * n and adam - sgd == 2 * (mom - sgd) and mom - sgd >= 4 * n
    assert adam - sgd < 2 * 4 * n * 1.2                               # two state arrays, modulo alignment
    small = binding.estimate_bytes(32, (1, 1, 96), "f32", layers, 8, "sgd")
    assert small < sgd                                                # fewer rows, fewer activations
    bf = binding.estimate_bytes(32, (1, 1, 96), "bf16", layers, 32, "sgd")
    assert bf > 8 * n and bf != sgd
    assert binding.estimate_bytes(32, (1, 1, 96), "f32", [("relu",)], 32, "sgd") == 0
    assert binding.estimate_bytes(32, (1, 1, 96), "f32", layers, 33, "sgd") == 0
