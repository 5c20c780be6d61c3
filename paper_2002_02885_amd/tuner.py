"""Hyperband and pack-aware Hyperband (paper Section 5, Algorithms 1 and 2) over the packed-training
library: an application-level driver, as the paper describes it.  Every decision (bracket plan,
grouping, successive halving) is taken by the library's host code and every training step runs in
its kernels; this module only walks the loops, builds the packs and carries checkpoints from rung to
rung.

Because packing is lossless, a configuration's losses do not depend on what it is packed with: all
grouping policies return the same winner and the same losses, and differ only in running time.

Readings (the text leaves them open): a resource unit is `steps_per_unit` training steps; a rung
resumes its survivors from their checkpoints (weights, optimiser state, step count); the
intermediate loss of a configuration is the mean training loss over the last `loss_window` steps
of the rung; step t of every configuration reads the rows that start at (t * max_batch) modulo
(n - max_batch) of the dataset and a configuration with a smaller batch takes the leading rows, so
that the data a configuration sees does not depend on its group.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np

from . import binding

BATCH_SIZES = [20, 25, 30, 35, 40, 45, 50, 55, 60, 65, 70]
OPTIMIZERS = ["adam", "sgd", "adagrad", "momentum"]
LEARNING_RATES = [0.000001, 0.00001, 0.0001, 0.001, 0.01, 0.1]
ACTIVATIONS = ["sigmoid", "leaky_relu", "tanh", "relu"]
CATEGORICAL = [0, 1, 0, 1]          # batch size and learning rate are ordered, optimiser and activation are not
POLICIES = ("none", "knn", "random", "batchsize")


def all_configurations():
    """The search space of the paper's evaluation (Table 3) as index tuples."""
    import itertools
    axes = (BATCH_SIZES, OPTIMIZERS, LEARNING_RATES, ACTIVATIONS)
    return list(itertools.product(*(range(len(axis)) for axis in axes)))


def mlp_family(hidden: Sequence[int], n_classes: int) -> Callable[[str], list]:
    """Architecture of a trial as a function of its activation."""
    def layers(activation: str) -> list:
        out = []
        for h in hidden:
            out += [("linear", int(h)), (activation,)]
        return out + [("linear", n_classes)]
    return layers


@dataclass
class Trial:
    cfg: tuple
    weights: np.ndarray
    opt_state: list = field(default_factory=list)
    steps_done: int = 0
    loss: float = float("inf")

    @property
    def batch(self):
        return BATCH_SIZES[self.cfg[0]]

    @property
    def optimizer(self):
        return OPTIMIZERS[self.cfg[1]]

    @property
    def lr(self):
        return LEARNING_RATES[self.cfg[2]]

    @property
    def activation(self):
        return ACTIVATIONS[self.cfg[3]]


class Tuner:
    def __init__(self, data_ptr: int, labels_ptr: int, n_samples: int, in_shape, dtype: str, family, init_weights,
                 steps_per_unit: int = 10, loss_window: int = 4, policy: str = "knn", capacity_bytes: int = 1 << 30,
                 threshold: int = 4, random_m: int = 8, seed: int = 0, sync: Optional[Callable[[], None]] = None):
        """data_ptr / labels_ptr: device addresses of the dataset [n_samples, H, W, C] (pack dtype) and its
        int32 labels; family(activation) -> layer list; init_weights(cfg, layers) -> flat fp32 blob."""
        assert policy in POLICIES and n_samples > max(BATCH_SIZES)
        self.data_ptr, self.labels_ptr, self.n = data_ptr, labels_ptr, n_samples
        self.in_shape, self.dtype, self.family, self.init_weights = tuple(in_shape), dtype, family, init_weights
        self.steps_per_unit, self.loss_window = steps_per_unit, loss_window
        self.policy, self.capacity, self.threshold, self.random_m = policy, capacity_bytes, threshold, random_m
        self.rng = np.random.default_rng(np.random.PCG64(seed))
        self.row_bytes = int(np.prod(in_shape)) * (2 if dtype == "bf16" else 4)
        self.sync = sync or (lambda: None)
        self.train_seconds = 0.0
        self.packs_built = 0
        self.log = []

    # -- grouping (Algorithm 2: packed_group <- pack_opt(T)) ---------------------------------------
    def groups(self, trials: List[Trial]) -> List[List[int]]:
        T = len(trials)
        if self.policy == "none":
            return [[i] for i in range(T)]
        need = [binding.estimate_bytes(max(BATCH_SIZES), self.in_shape, self.dtype, self.family(t.activation), t.batch,
                                       t.optimizer) for t in trials]
        if self.policy == "knn":
            return binding.opt_knn([t.cfg for t in trials], CATEGORICAL, need, self.capacity, self.threshold, self.rng.random(T))
        if self.policy == "random":
            return binding.opt_random(T, self.random_m, self.rng.permutation(T))
        return binding.opt_batchsize([t.batch for t in trials], need, self.capacity)

    # -- one packed group trained up to steps_total -------------------------------------------------
    def train_group(self, trials: List[Trial], steps_total: int):
        B = max(t.batch for t in trials)
        pk = binding.Pack(B, self.in_shape, self.dtype, [self.family(t.activation) for t in trials], [t.batch for t in trials])
        self.packs_built += 1
        try:
            for k, t in enumerate(trials):
                pk.write_weights(k, t.weights)
                pk.set_optimizer(k, {"kind": t.optimizer})
                for slot, state in enumerate(t.opt_state):
                    pk.write_opt_state(k, slot, state, t.steps_done)
            lr = np.array([t.lr for t in trials], dtype=np.float32)
            start = trials[0].steps_done
            assert all(t.steps_done == start for t in trials)
            acc, cnt = np.zeros(len(trials)), 0
            span = self.n - max(BATCH_SIZES)
            for step in range(start, steps_total):
                row = (step * max(BATCH_SIZES)) % span
                pk.step(self.data_ptr + row * self.row_bytes, self.labels_ptr + row * 4, lr)
                if step >= steps_total - self.loss_window:
                    acc += pk.read_loss()
                    cnt += 1
            for k, t in enumerate(trials):
                t.weights = pk.read_weights(k)
                n_state = {"sgd": 0, "momentum": 1, "adagrad": 1, "adam": 2}[t.optimizer]
                t.opt_state = [pk.read_opt_state(k, s)[0] for s in range(n_state)]
                t.steps_done = steps_total
                if cnt:
                    t.loss = float(acc[k] / cnt)
        finally:
            pk.destroy()

    # -- Algorithms 1 / 2 -----------------------------------------------------------------------------
    def run(self, R: int, eta: int, sampled: Optional[List[List[tuple]]] = None):
        """sampled[j]: the configurations of bracket j (drawn here without replacement when not given).
        Returns (best configuration, its loss)."""
        space = all_configurations()
        best, best_loss = None, float("inf")
        for j, rungs in enumerate(binding.hyperband_plan(R, eta)):
            n0 = rungs[0][0]
            cfgs = sampled[j][:n0] if sampled is not None else [space[i] for i in self.rng.choice(len(space), size=min(n0, len(space)), replace=False)]
            trials = [Trial(tuple(c), self.init_weights(tuple(c), self.family(ACTIVATIONS[c[3]]))) for c in cfgs]
            for i, (n_i, r_i) in enumerate(rungs):
                trials = trials[:n_i]
                groups = self.groups(trials)
                self.sync()
                t0 = time.perf_counter()
                for g in groups:
                    self.train_group([trials[k] for k in g], r_i * self.steps_per_unit)
                self.sync()
                self.train_seconds += time.perf_counter() - t0
                losses = [t.loss for t in trials]
                self.log.append({"bracket": j, "rung": i, "configs": [t.cfg for t in trials], "groups": groups,
                                 "losses": losses, "r": r_i})
                for t in trials:
                    if np.isfinite(t.loss) and t.loss < best_loss:    # a diverged run never becomes the winner
                        best, best_loss = t.cfg, t.loss
                if i + 1 < len(rungs):
                    keep = binding.halving_keep(losses, max(n_i // eta, 1))
                    trials = [trials[k] for k in keep]
        return best, best_loss
