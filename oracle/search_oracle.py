"""CPU oracle for the pack-aware hyper-parameter search (paper Section 5).  TEST INFRASTRUCTURE
ONLY: nothing in the product path may import, call or link this file.

What it covers, each in the order and notation of the text:
  * the search space of the evaluation (Section 5.3, Table 3): 11 batch sizes x 4 optimisers x
    6 learning rates x 4 activations = 1056 configurations;
  * the distance between two configurations (Section 5.2): numeric hyper-parameters (batch size,
    learning rate) contribute the difference of their INDICES in the table, categorical ones
    (optimiser, activation) 0 if equal and 1 if not;
  * pack_opt, the nearest-neighbour heuristic (Section 5.2): pick a random configuration among
    those not yet grouped as centroid, add the configurations most similar to it, nearest first,
    until the device memory is used up; a similarity threshold bounds how far a configuration may
    be from the centroid; repeat until every configuration is in a group;
  * the two comparison heuristics (Section 5.3): Random Pack (m randomly chosen configurations per
    group) and Batch-size Pack (only equal batch sizes, greedily until the memory is full);
  * Hyperband's outer and inner loops (Section 5.1, Algorithm 1; the bracket sizes come from the
    Hyperband paper the text cites, Li et al. 2017, Algorithm 1) and the pack-aware variant
    (Section 5.2, Algorithm 2), which differs only in training the configurations of a rung in
    the groups pack_opt returns.

Readings where the text is silent or at odds with itself:
  * the text calls the distance "Euclid" but the worked example (A = [20, SGD, 0.01, ReLU],
    B = [40, Adagrad, 0.01, ReLU], distance 5) is the SUM of the per-dimension differences
    (4 index steps of batch size + 1 for the optimiser); the Euclidean value would be sqrt(17).
    The printed number is followed: the distance is the sum of absolute differences;
  * ties between equally distant configurations go to the one that comes first in the list;
  * a configuration joins a group only if its distance to the centroid is <= the threshold and
    the group's memory still has room for it; a nearer one that does not fit is skipped and a
    farther, smaller one may still join ("until the device runs out of memory" = nothing more fits);
  * every random choice is an input: the centroid of round j is element floor(u_j * remaining) of
    the not-yet-grouped configurations in list order, with u_j in [0, 1) supplied by the caller;
    Random Pack takes a permutation; Hyperband takes the sampled configurations of each bracket;
  * the memory a configuration needs is supplied by the caller, one number per configuration
    (the paper probes for out-of-memory; the library computes the number from the model);
  * Hyperband keeps floor(n_i / eta) configurations after rung i, those with the smallest loss,
    the earlier one on ties; a rung trains for r_i = r * eta^i resource units in total.
"""
from __future__ import annotations

import math

BATCH_SIZES = [20, 25, 30, 35, 40, 45, 50, 55, 60, 65, 70]
OPTIMIZERS = ["adam", "sgd", "adagrad", "momentum"]
LEARNING_RATES = [0.000001, 0.00001, 0.0001, 0.001, 0.01, 0.1]
ACTIVATIONS = ["sigmoid", "leaky_relu", "tanh", "relu"]
# a configuration is a tuple of indices (batch size, optimiser, learning rate, activation)
CATEGORICAL = (False, True, False, True)


def all_configurations():
    return [(b, o, l, a) for b in range(len(BATCH_SIZES)) for o in range(len(OPTIMIZERS))
            for l in range(len(LEARNING_RATES)) for a in range(len(ACTIVATIONS))]


def configuration(batch, optimizer, lr, activation):
    return (BATCH_SIZES.index(batch), OPTIMIZERS.index(optimizer), LEARNING_RATES.index(lr), ACTIVATIONS.index(activation))


def distance(a, b, categorical=CATEGORICAL):
    d = 0
    for x, y, cat in zip(a, b, categorical):
        if cat:
            d += 0 if x == y else 1
        else:
            d += abs(x - y)
    return d


def pack_opt_knn(configs, need, capacity, threshold, draws, categorical=CATEGORICAL):
    """Groups of indices into `configs`.  need[i]: memory of configuration i; capacity: memory of
    the device; draws: one number in [0, 1) per group formed (at most len(configs) are used)."""
    remaining = list(range(len(configs)))
    groups = []
    draws = iter(draws)
    while remaining:
        u = next(draws)
        centroid = remaining[int(math.floor(u * len(remaining)))]
        remaining.remove(centroid)
        group, used = [centroid], need[centroid]
        by_distance = sorted(remaining, key=lambda i: distance(configs[centroid], configs[i], categorical))
        for i in by_distance:                                   # nearest first; sorted() keeps list order on ties
            if distance(configs[centroid], configs[i], categorical) > threshold:
                break
            if used + need[i] <= capacity:
                group.append(i)
                used += need[i]
        for i in group[1:]:
            remaining.remove(i)
        groups.append(group)
    return groups


def pack_random(n, m, perm):
    """Random Pack: the configurations in the order of the permutation, m per group."""
    if sorted(perm) != list(range(n)) or m < 1:
        raise ValueError("perm must be a permutation of range(n) and m >= 1")
    return [list(perm[s:s + m]) for s in range(0, n, m)]


def pack_batchsize(configs, need, capacity):
    """Batch-size Pack: only configurations with the same batch size share a group; within a batch
    size, in list order, a group is filled until the next configuration does not fit."""
    groups = []
    for b in sorted(set(c[0] for c in configs)):
        group, used = [], 0
        for i, c in enumerate(configs):
            if c[0] != b:
                continue
            if group and used + need[i] > capacity:
                groups.append(group)
                group, used = [], 0
            group.append(i)
            used += need[i]
        if group:
            groups.append(group)
    return groups


def hyperband_brackets(R, eta):
    """Li et al. 2017, Algorithm 1: for s = s_max .. 0 a bracket of rungs (n_i, r_i)."""
    s_max = 0
    while eta ** (s_max + 1) <= R:                              # floor(log_eta R) in integers
        s_max += 1
    B = (s_max + 1) * R
    brackets = []
    for s in range(s_max, -1, -1):
        n = -((-B * eta ** s) // (R * (s + 1)))                 # ceil(B/R * eta^s / (s+1))
        rungs = []
        for i in range(s + 1):
            n_i = n // eta ** i                                 # floor(n * eta^-i)
            r_i = R * eta ** i // eta ** s                      # r * eta^i with r = R * eta^-s
            rungs.append((n_i, r_i))
        brackets.append(rungs)
    return brackets


def keep_best(losses, keep):
    """Indices of the `keep` smallest losses, the earlier one on ties, in increasing index order.
    A loss that is not a number (a diverged run) ranks after every number, +inf included: Section 5.1
    keeps the best fraction, and a run without a loss cannot be among the best."""
    order = sorted(range(len(losses)), key=lambda i: (1, 0.0, i) if math.isnan(losses[i]) else (0, losses[i], i))
    return sorted(order[:keep])


def hyperband(R, eta, sampled, train, group_fn=None):
    """Algorithm 1 (group_fn None: every configuration alone) and Algorithm 2 (group_fn = a
    pack_opt).  sampled[j]: the configurations drawn for bracket j (at least n of them);
    train(groups_of_configs, r) -> one loss per configuration in the same nesting, after training
    for r resource units in total.  Returns (best configuration, its loss, log of rungs)."""
    best, best_loss, log = None, float("inf"), []
    for j, rungs in enumerate(hyperband_brackets(R, eta)):
        T = list(sampled[j][:rungs[0][0]])
        for i, (n_i, r_i) in enumerate(rungs):
            T = T[:n_i]
            groups = [[k] for k in range(len(T))] if group_fn is None else group_fn(T)
            nested = train([[T[k] for k in g] for g in groups], r_i)
            losses = [None] * len(T)
            for g, ls in zip(groups, nested):
                for k, l in zip(g, ls):
                    losses[k] = l
            log.append({"bracket": j, "rung": i, "configs": list(T), "groups": groups, "losses": losses, "r": r_i})
            for k, l in enumerate(losses):
                if l < best_loss:
                    best, best_loss = T[k], l
            T = [T[k] for k in keep_best(losses, max(n_i // eta, 1) if i + 1 < len(rungs) else len(T))]
    return best, best_loss, log
