"""Pack-aware Hyperband (paper Section 5, Algorithms 1 and 2) end to end on the GPU, on a small
learnable synthetic dataset: all grouping policies must return the same losses and the same winner
as plain Hyperband (packing is lossless), and every loss must be the one the oracle reaches by
training that configuration alone, from scratch, on the same rows."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pack_oracle as po
from oracle import search_oracle as so
from paper_2002_02885_amd import binding, tuner

pytestmark = pytest.mark.gpu

IN_SHAPE, N, UNIT, WINDOW = (1, 1, 96), 1500, 4, 2


def _init(cfg, layers):
    seed = 7919 + ((cfg[0] * 4 + cfg[1]) * 6 + cfg[2]) * 4 + cfg[3]
    return wl.draw_weights(np.random.default_rng(np.random.PCG64(seed)), layers, IN_SHAPE, wl.F32)


def _run(policy, data, labels, sampled, R, eta):
    t = tuner.Tuner(data.data_ptr(), labels.data_ptr(), N, IN_SHAPE, wl.F32, tuner.mlp_family([48], 10), _init,
                    steps_per_unit=UNIT, loss_window=WINDOW, policy=policy, capacity_bytes=400_000, threshold=5,
                    random_m=4, seed=1, sync=torch.cuda.synchronize)
    best = t.run(R, eta, sampled)
    return best, t


def test_space_and_tables_match_the_oracles():
    assert tuner.all_configurations() == so.all_configurations()
    assert (tuner.BATCH_SIZES, tuner.OPTIMIZERS, tuner.LEARNING_RATES, tuner.ACTIVATIONS) == \
           (so.BATCH_SIZES, so.OPTIMIZERS, so.LEARNING_RATES, so.ACTIVATIONS)
    assert [bool(c) for c in tuner.CATEGORICAL] == list(so.CATEGORICAL)


def test_all_policies_find_the_same_winner_with_the_same_losses_and_match_the_oracle():
    R, eta = 9, 3
    X, Y = wl.labelled_dataset(7, N, IN_SHAPE)
    data, labels = torch.from_numpy(X).cuda().contiguous(), torch.from_numpy(Y).cuda().contiguous()
    space = so.all_configurations()
    rng = np.random.default_rng(11)
    sampled = [[space[i] for i in rng.choice(len(space), size=rungs[0][0], replace=False)]
               for rungs in so.hyperband_brackets(R, eta)]
    (best, best_loss), plain = _run("none", data, labels, sampled, R, eta)
    assert [len(e["configs"]) for e in plain.log] == [n for rungs in so.hyperband_brackets(R, eta) for n, _ in rungs]
    for policy in ("knn", "random", "batchsize"):
        (b, l), t = _run(policy, data, labels, sampled, R, eta)
        assert (b, l) == (best, best_loss), policy
        assert [(e["configs"], e["losses"]) for e in t.log] == [(e["configs"], e["losses"]) for e in plain.log], policy
        assert t.packs_built < plain.packs_built, policy
        for e in t.log:
            assert sorted(i for g in e["groups"] for i in g) == list(range(len(e["configs"])))
            if policy == "batchsize":
                assert all(len(set(e["configs"][i][0] for i in g)) == 1 for g in e["groups"])
            if policy == "random":
                assert all(len(g) <= 4 for g in e["groups"])
            if policy == "knn":
                need = [binding.estimate_bytes(70, IN_SHAPE, wl.F32, tuner.mlp_family([48], 10)(so.ACTIVATIONS[c[3]]),
                                               so.BATCH_SIZES[c[0]], so.OPTIMIZERS[c[1]]) for c in e["configs"]]
                assert all(sum(need[i] for i in g) <= 400_000 for g in e["groups"])
    # the oracle: every configuration of every rung alone, from scratch, in float64
    tol = 1e-4
    span = N - max(so.BATCH_SIZES)
    for j, rungs in enumerate(so.hyperband_brackets(R, eta)):
        entries = [e for e in plain.log if e["bracket"] == j]
        for i, e in enumerate(entries):
            steps = e["r"] * UNIT
            ref = []
            for cfg in e["configs"]:
                layers = tuner.mlp_family([48], 10)(so.ACTIVATIONS[cfg[3]])
                net = po.Model(layers, IN_SHAPE, _init(cfg, layers).astype(np.float64), "exact", opt={"kind": so.OPTIMIZERS[cfg[1]]})
                b, lr, tail = so.BATCH_SIZES[cfg[0]], so.LEARNING_RATES[cfg[2]], []
                for s in range(steps):
                    row = (s * max(so.BATCH_SIZES)) % span
                    l = net.sgd_step(X[row:row + b].astype(np.float64), Y[row:row + b], lr)[0]
                    if s >= steps - WINDOW:
                        tail.append(l)
                ref.append(float(np.mean(tail)))
            for got, want, cfg in zip(e["losses"], ref, e["configs"]):
                assert abs(got - want) <= tol * abs(want), (j, i, cfg, got, want)
            if i + 1 < len(entries):
                keep = max(len(ref) // eta, 1)
                kept = set(entries[i + 1]["configs"])
                cut = sorted(ref)[keep - 1]
                for cfg, l in zip(e["configs"], ref):
                    if cfg in kept:
                        assert l <= cut * (1 + 2 * tol), (j, i, cfg)
                    else:
                        assert l >= cut * (1 - 2 * tol), (j, i, cfg)
    ref_best = min(l for e in plain.log for l in e["losses"])
    assert best_loss == ref_best


def test_memory_model_tracks_what_a_pack_really_allocates():
    """pack_estimate_bytes per member, summed, against pack_device_bytes of the pack that holds them
    (which adds what members share: workspace, problem tables, small fixed buffers)."""
    cases = [(wl.config2(B=64, D=512, hidden=(256, 128), K=6, steps=1), ["sgd", "adam", "momentum", "sgd", "adagrad", "adam"]),
             (wl.config3(K=3, B=8, size=16, widths=(16, 32, 32), steps=1), ["sgd", "sgd", "sgd"]),
             (wl.config4(K=8, B=64, D=256, width_choices=(32, 96, 200), steps=1), ["sgd"] * 8)]
    for w, opts in cases:
        pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
        try:
            for k, o in enumerate(opts):
                pk.set_optimizer(k, {"kind": o})
            real = pk.device_bytes()
        finally:
            pk.destroy()
        est = sum(binding.estimate_bytes(w.B, w.in_shape, w.dtype, w.models[k], w.batch[k], opts[k]) for k in range(w.K))
        # state arrays are arena-shaped: a pack with one Adam member holds both arrays for every member
        n_state = max({"sgd": 0, "momentum": 1, "adagrad": 1, "adam": 2}[o] for o in opts)
        est_upper = sum(binding.estimate_bytes(w.B, w.in_shape, w.dtype, w.models[k], w.batch[k],
                                               ["sgd", "momentum", "adam"][n_state]) for k in range(w.K))
        assert est <= real, (w.name, est, real)
        assert real <= 1.25 * est_upper + (2 << 20), (w.name, est_upper, real)
        print(f"\n{w.name}: estimate {est / 1e6:.2f} MB (arena-shaped state: {est_upper / 1e6:.2f} MB), allocated {real / 1e6:.2f} MB")
