"""Pins for the optimisers of the oracle (paper Table 3: Adam, SGD, Adagrad, Momentum; state stored
with the model, Section 2.2).  Three independent kinds of evidence: closed forms under a constant
gradient, an independent optimiser library on random gradient sequences, and whole training runs
against an independent autograd + optimiser library."""
import math

import numpy as np
import pytest
import torch

from oracle import pack_oracle as po

RNG = lambda s: np.random.Generator(np.random.PCG64(s))

OPTS = {
    "sgd": {"kind": "sgd"},
    "momentum": {"kind": "momentum", "mu": 0.9},
    "momentum_mu05": {"kind": "momentum", "mu": 0.5},
    "adagrad": {"kind": "adagrad", "acc0": 0.1},
    "adam": {"kind": "adam", "beta1": 0.9, "beta2": 0.999, "eps": 1e-8},
    "adam_other": {"kind": "adam", "beta1": 0.8, "beta2": 0.95, "eps": 1e-6},
}


def _run(opt, w0, grads, lr):
    w = np.array(w0, dtype=np.float64)
    st = po.new_opt_state(opt, w.shape)
    for t, g in enumerate(grads, start=1):
        po.apply_update(opt, w, np.asarray(g, dtype=np.float64), st, lr, t)
    return w, st


def test_closed_forms_under_a_constant_gradient():
    g, lr, w0, n = 0.37, 0.05, 1.25, 9
    grads = [np.array([g])] * n
    # plain SGD: a straight line
    w, _ = _run(OPTS["sgd"], [w0], grads, lr)
    assert abs(w[0] - (w0 - n * lr * g)) < 1e-15
    # momentum: acc_i = g (1 - mu^i) / (1 - mu)
    for mu in (0.9, 0.5):
        w, st = _run({"kind": "momentum", "mu": mu}, [w0], grads, lr)
        want = w0 - lr * g * sum((1 - mu ** i) / (1 - mu) for i in range(1, n + 1))
        assert abs(w[0] - want) < 1e-14 and abs(st[0][0] - g * (1 - mu ** n) / (1 - mu)) < 1e-14
    # adagrad: acc_i = acc0 + i g^2
    w, st = _run({"kind": "adagrad", "acc0": 0.1}, [w0], grads, lr)
    want = w0 - lr * sum(g / math.sqrt(0.1 + i * g * g) for i in range(1, n + 1))
    assert abs(w[0] - want) < 1e-14 and abs(st[0][0] - (0.1 + n * g * g)) < 1e-14
    # adam: the bias-corrected moments of a constant are the constant and its square, so every
    # step moves by lr * g / (|g| + eps) whatever beta1 and beta2 are
    for key in ("adam", "adam_other"):
        o = OPTS[key]
        w, _ = _run(o, [w0], grads, lr)
        assert abs(w[0] - (w0 - n * lr * g / (abs(g) + o["eps"]))) < 1e-13
    # ... and a sign flip of the gradient flips the direction
    w, _ = _run(OPTS["adam"], [w0], [np.array([-g])] * n, lr)
    assert w[0] > w0


def test_adam_first_step_is_lr_times_sign():
    r = RNG(3)
    g = r.standard_normal(50)
    w, _ = _run(OPTS["adam"], np.zeros(50), [g], 0.01)
    assert np.allclose(w, -0.01 * np.sign(g), rtol=0, atol=1e-8)


def _torch_opt(key, params, lr):
    o = OPTS[key]
    if o["kind"] == "sgd":
        return torch.optim.SGD(params, lr=lr)
    if o["kind"] == "momentum":
        return torch.optim.SGD(params, lr=lr, momentum=o["mu"])
    if o["kind"] == "adagrad":
        return torch.optim.Adagrad(params, lr=lr, initial_accumulator_value=o["acc0"], eps=0.0)
    return torch.optim.Adam(params, lr=lr, betas=(o["beta1"], o["beta2"]), eps=o["eps"])


@pytest.mark.parametrize("key", sorted(OPTS))
def test_update_rule_matches_independent_library_on_random_gradients(key):
    r = RNG(11)
    w0 = r.standard_normal((4, 3))
    grads = [r.standard_normal((4, 3)) * 10 ** r.uniform(-3, 1) for _ in range(7)]
    w, _ = _run(OPTS[key], w0, grads, 0.03)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = _torch_opt(key, [p], 0.03)
    for g in grads:
        p.grad = torch.from_numpy(g.copy())
        opt.step()
    assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14), np.max(np.abs(w - p.detach().numpy()))


def test_the_library_pin_notices_a_dropped_bias_correction():
    """Negative control: Adam without the 1/(1-beta^t) factors is far outside the pin's tolerance."""
    r = RNG(12)
    w0 = r.standard_normal(6)
    grads = [r.standard_normal(6) for _ in range(5)]
    o = OPTS["adam"]
    w = w0.copy()
    m = np.zeros(6); v = np.zeros(6)
    for g in grads:                                   # the mutated rule
        m = o["beta1"] * m + (1 - o["beta1"]) * g
        v = o["beta2"] * v + (1 - o["beta2"]) * g * g
        w -= 0.03 * m / (np.sqrt(v) + o["eps"])
    good, _ = _run(o, w0, grads, 0.03)
    assert np.max(np.abs(w - good)) > 1e-3


LAYERS = {
    "mlp_tanh": ((1, 1, 6), [("linear", 5), ("tanh",), ("linear", 4), ("sigmoid",), ("linear", 3)]),
    "cnn_leaky": ((5, 5, 2), [("conv3x3", 3, 1), ("leaky_relu",), ("conv3x3", 4, 2), ("relu",), ("gap",), ("linear", 3)]),
}


@pytest.mark.parametrize("net", sorted(LAYERS))
@pytest.mark.parametrize("key", ["momentum", "adagrad", "adam"])
def test_training_runs_match_independent_autograd_and_optimiser(net, key):
    from test_oracle_pins import _torch_loss
    import workloads as wl
    in_shape, layers = LAYERS[net]
    r = RNG(21)
    blob = r.standard_normal(wl.num_params(layers, in_shape)) * 0.6
    x = r.standard_normal((5,) + in_shape)
    y = r.integers(0, 3, 5)
    steps, lr = 4, 0.05
    model = po.Model(layers, in_shape, blob, opt=OPTS[key])
    losses = [model.sgd_step(x, y, lr)[0] for _ in range(steps)]
    bt = torch.nn.Parameter(torch.from_numpy(blob.copy()))
    opt = _torch_opt(key, [bt], lr)
    for t in range(steps):
        opt.zero_grad()
        loss_t, _ = _torch_loss(layers, in_shape, bt, x, y)
        assert abs(loss_t.item() - losses[t]) < 1e-10, (t, loss_t.item(), losses[t])
        loss_t.backward()
        opt.step()
    assert np.allclose(model.blob(), bt.detach().numpy(), rtol=1e-9, atol=1e-11)


def test_members_keep_their_own_optimiser_and_state():
    """Paper Table 2, "Optimizer: Different": members of one pack may use different optimisers; each
    member's trajectory is that of the member trained alone."""
    import workloads as wl
    in_shape = (1, 1, 5)
    layers = [("linear", 4), ("relu",), ("linear", 3)]
    r = RNG(31)
    blobs = [r.standard_normal(wl.num_params(layers, in_shape)) * 0.5 for _ in range(3)]
    x = r.standard_normal((6,) + in_shape)
    y = r.integers(0, 3, 6)
    opts = [OPTS["adam"], OPTS["sgd"], OPTS["momentum"]]
    out = po.train_pack([layers] * 3, in_shape, blobs, [6, 4, 6], [0.01, 0.1, 0.05], x, y, 3, optimizers=opts)
    for k in range(3):
        solo = po.train_pack([layers], in_shape, [blobs[k]], [[6, 4, 6][k]], [[0.01, 0.1, 0.05][k]], x, y, 3,
                             optimizers=[opts[k]])
        assert np.array_equal(out["blobs"][k], solo["blobs"][0])
        assert np.array_equal(out["loss"][:, k], solo["loss"][:, 0])
    # the state travels with the model: Adam's step counter and moments after three steps
    assert out["nets"][0].t == 3 and np.all(out["nets"][0].opt_state_blob(1) >= 0)
