"""Pins of the search oracle (paper Section 5): the printed numbers, metric properties, closed
forms of the Hyperband brackets, invariants and small brute-force cases of the grouping heuristics."""
import itertools
import os

import numpy as np
import pytest

from oracle import search_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "search_worked_examples.txt")


def _gold():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_the_papers_distance_example_and_space_size():
    g = _gold()
    a = so.configuration(20, "sgd", 0.01, "relu")
    b = so.configuration(40, "adagrad", 0.01, "relu")
    assert so.distance(a, b) == g["distance_A_B"]
    # the Euclidean reading of the same example would give sqrt(17), not the printed 5
    assert not np.isclose(np.sqrt(sum((x - y) ** 2 if not c else (x != y) for x, y, c in zip(a, b, so.CATEGORICAL))), 5.0)
    confs = so.all_configurations()
    assert len(confs) == g["configurations"] and len(set(confs)) == len(confs)


def test_distance_is_a_metric_and_matches_an_array_formulation():
    confs = so.all_configurations()
    rng = np.random.default_rng(0)
    pick = [confs[i] for i in rng.choice(len(confs), size=40, replace=False)]
    arr = np.array(pick)
    cat = np.array(so.CATEGORICAL)
    for i, j in itertools.product(range(40), repeat=2):
        want = int(np.abs(arr[i, ~cat] - arr[j, ~cat]).sum() + (arr[i, cat] != arr[j, cat]).sum())
        assert so.distance(pick[i], pick[j]) == want == so.distance(pick[j], pick[i])
        assert (want == 0) == (pick[i] == pick[j])
    for i, j, k in rng.integers(0, 40, size=(300, 3)):
        assert so.distance(pick[i], pick[k]) <= so.distance(pick[i], pick[j]) + so.distance(pick[j], pick[k])


def test_hyperband_brackets_closed_forms():
    g = _gold()
    R, eta = int(g["R"]), int(g["eta"])
    br = so.hyperband_brackets(R, eta)
    assert len(br) == 5                                          # s_max = log_3 81 = 4
    B = 5 * R
    assert br[0] == [(81, 1), (27, 3), (9, 9), (3, 27), (1, 81)]   # n = 81 halves by eta, r grows by eta
    assert sum(n * r for n, r in br[0]) == B
    for s, rungs in zip(range(4, -1, -1), br):
        assert len(rungs) == s + 1 and rungs[-1][1] == R and rungs[0][1] == R // eta ** s
        assert rungs[0][0] == -(-5 * eta ** s // (s + 1))        # ceil((s_max+1) eta^s / (s+1))
        for (n0, r0), (n1, r1) in zip(rungs, rungs[1:]):
            assert n1 == n0 // eta and r1 == r0 * eta
        assert sum(n * r for n, r in rungs) <= B
    assert br[-1] == [(5, 81)]
    assert so.hyperband_brackets(1, 3) == [[(1, 1)]]
    assert so.hyperband_brackets(9, 3) == [[(9, 1), (3, 3), (1, 9)], [(5, 3), (1, 9)], [(3, 9)]]


def _is_partition(groups, n):
    flat = [i for g in groups for i in g]
    return sorted(flat) == list(range(n))


def test_knn_grouping_invariants_on_random_inputs():
    confs_all = so.all_configurations()
    rng = np.random.default_rng(1)
    for trial in range(60):
        T = int(rng.integers(1, 40))
        confs = [confs_all[i] for i in rng.integers(0, len(confs_all), size=T)]     # duplicates allowed
        need = [int(v) for v in rng.integers(1, 10, size=T)]
        capacity = int(rng.integers(5, 40))
        threshold = int(rng.integers(0, 12))
        draws = rng.random(T)
        groups = so.pack_opt_knn(confs, need, capacity, threshold, draws)
        assert _is_partition(groups, T)
        for g in groups:
            c = g[0]
            assert sum(need[i] for i in g) <= max(capacity, need[c])
            ds = [so.distance(confs[c], confs[i]) for i in g[1:]]
            assert all(d <= threshold for d in ds) and ds == sorted(ds)      # nearest first


def test_knn_grouping_uniform_memory_is_the_k_nearest_within_the_threshold():
    confs_all = so.all_configurations()
    rng = np.random.default_rng(2)
    for trial in range(40):
        T = int(rng.integers(2, 25))
        confs = [confs_all[i] for i in rng.choice(len(confs_all), size=T, replace=False)]
        per_group = int(rng.integers(1, 6))
        threshold = int(rng.integers(0, 10))
        draws = list(rng.random(T))
        groups = so.pack_opt_knn(confs, [1] * T, per_group, threshold, draws)
        remaining = list(range(T))
        for g, u in zip(groups, draws):
            c = remaining[int(u * len(remaining))]
            others = [i for i in remaining if i != c]
            d = np.array([so.distance(confs[c], confs[i]) for i in others])
            order = np.argsort(d, kind="stable")
            want = [c] + [others[j] for j in order[:per_group - 1] if d[j] <= threshold]
            assert g == want
            remaining = [i for i in remaining if i not in g]
        assert not remaining


def test_knn_grouping_hand_worked_case():
    # five configurations on a line (only the batch-size index differs): 0, 1, 2, 6, 7
    confs = [(0, 1, 2, 3), (1, 1, 2, 3), (2, 1, 2, 3), (6, 1, 2, 3), (7, 1, 2, 3)]
    # centroid draw 0.5 of 5 remaining -> element 2; threshold 2 admits 1 (d=1) then 0 (d=2); memory 3 holds all
    # then 2 remain (3, 4): draw 0.0 -> 3, which takes 4 (d=1)
    assert so.pack_opt_knn(confs, [1] * 5, 3, 2, [0.5, 0.0]) == [[2, 1, 0], [3, 4]]
    # memory for two only: the nearer one wins; a skipped big one does not block a smaller, farther one
    assert so.pack_opt_knn(confs, [1] * 5, 2, 2, [0.5, 0.0, 0.0]) == [[2, 1], [0], [3, 4]]
    assert so.pack_opt_knn(confs, [1, 5, 1, 1, 1], 3, 2, [0.5, 0.0, 0.0]) == [[2, 0], [1], [3, 4]]
    # threshold 0: only identical configurations share a group; a centroid larger than the device still runs alone
    assert so.pack_opt_knn(confs + [confs[0]], [9] + [1] * 5, 3, 0, [0.0] * 6) == [[0], [1], [2], [3], [4], [5]]
    assert so.pack_opt_knn(confs + [confs[0]], [1] * 6, 3, 0, [0.0] * 6) == [[0, 5], [1], [2], [3], [4]]


def test_comparison_heuristics():
    confs_all = so.all_configurations()
    rng = np.random.default_rng(3)
    confs = [confs_all[i] for i in rng.choice(len(confs_all), size=50, replace=False)]
    perm = [int(i) for i in rng.permutation(50)]
    groups = so.pack_random(50, 8, perm)
    assert _is_partition(groups, 50) and [len(g) for g in groups] == [8] * 6 + [2]
    assert [i for g in groups for i in g] == perm
    groups = so.pack_batchsize(confs, [2] * 50, 7)                  # three members of need 2 fit
    assert _is_partition(groups, 50)
    for g in groups:
        assert len(set(confs[i][0] for i in g)) == 1 and len(g) <= 3 and g == sorted(g)
    for b in set(c[0] for c in confs):
        count = sum(1 for c in confs if c[0] == b)
        assert sum(1 for g in groups if confs[g[0]][0] == b) == -(-count // 3)
    with pytest.raises(ValueError):
        so.pack_random(5, 2, [0, 1, 2, 3, 3])


def test_keep_best_breaks_ties_by_position():
    assert so.keep_best([0.5, 0.1, 0.5, 0.1, 0.9], 3) == [0, 1, 3]
    assert so.keep_best([3.0, 2.0, 1.0], 1) == [2]


def test_keep_best_ranks_diverged_runs_last():
    nan, inf = float("nan"), float("inf")
    # a finite loss always survives ahead of inf, and inf ahead of NaN, wherever they sit
    assert so.keep_best([nan, 5.0, inf, 1.0], 2) == [1, 3]
    assert so.keep_best([nan, 5.0, inf, 1.0], 3) == [1, 2, 3]
    assert so.keep_best([nan, nan, 2.0], 1) == [2]
    assert so.keep_best([nan, nan, 2.0], 2) == [0, 2]
    assert so.keep_best([inf, nan, inf], 2) == [0, 2]


def test_hyperband_returns_the_best_sampled_configuration_and_grouping_does_not_change_it():
    confs = so.all_configurations()
    rng = np.random.default_rng(4)
    target = (5, 2, 3, 1)
    score = {c: so.distance(c, target) + 0.001 * i for i, c in enumerate(confs)}     # strictly ordered

    def train(nested, r):
        return [[score[c] / (1.0 + 0.0 * r) for c in g] for g in nested]

    brackets = so.hyperband_brackets(81, 3)
    sampled = [[confs[i] for i in rng.choice(len(confs), size=rungs[0][0], replace=False)] for rungs in brackets]
    best, loss, log = so.hyperband(81, 3, sampled, train)
    everything = [c for s in sampled for c in s]
    assert best == min(everything, key=lambda c: score[c]) and loss == score[best]
    assert [len(e["configs"]) for e in log[:5]] == [81, 27, 9, 3, 1]
    need = {c: 1 + c[0] for c in confs}
    draws = list(rng.random(2000))

    def knn(T):
        return so.pack_opt_knn(T, [need[c] for c in T], 24, 4, draws)

    best2, loss2, log2 = so.hyperband(81, 3, sampled, train, group_fn=knn)
    assert (best2, loss2) == (best, loss)
    assert [e["losses"] for e in log2] == [e["losses"] for e in log]
    assert any(len(g) > 1 for e in log2 for g in e["groups"])
