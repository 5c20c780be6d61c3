"""The comparison helpers of the GPU parity tests, exercised on the CPU: the oracle stands in for
the device run, and mistakes are planted in the oracle's output to see the gate close."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu


def _as_gpu(ref):
    return {"loss": ref["loss"].copy(), "grads": [g.astype(np.float32) for g in ref["grads"][0]],
            "blobs": [b.astype(np.float32) for b in ref["blobs"]]}


def test_gate_accepts_the_oracle_and_rejects_planted_mistakes():
    w = wl.config1(B=8, D=24, hidden=12)
    ref = pu.run_oracle(w, 2)
    good = _as_gpu(ref)
    worst = pu.compare(w, good, ref, 1e-4)
    assert worst["grad_inf"] < 1e-6 and worst["disp_l2"] < 1e-4 + 1e-3
    for plant in ("grad_scale", "grad_transpose", "loss", "bias_sign", "lr_swapped"):
        bad = _as_gpu(ref)
        if plant == "grad_scale":
            bad["grads"][1][:10] *= 1.001
        elif plant == "grad_transpose":
            Wg = bad["grads"][0][:12 * 24].reshape(12, 24)
            bad["grads"][0][:12 * 24] = Wg.T.reshape(-1)
        elif plant == "loss":
            bad["loss"][1, 0] *= 1.0002
        elif plant == "bias_sign":
            s = dict(pu.tensor_slices(w.models[0], w.in_shape))["linear0.b"]
            bad["blobs"][0][s] = 2 * w.weights[0][s] - bad["blobs"][0][s]
        elif plant == "lr_swapped":
            bad["blobs"][0] = (w.weights[0] + (ref["blobs"][0] - w.weights[0]) * 10).astype(np.float32)
        with pytest.raises(AssertionError):
            pu.compare(w, bad, ref, 1e-4)


def test_ill_conditioned_items_are_reported_not_hidden():
    w = wl.config1(B=8, D=24, hidden=12)
    ref = pu.run_oracle(w, 1)
    bad = _as_gpu(ref)
    bad["grads"][0][:5] *= 1.01
    key = ("grad_l2", 0, "linear0.W")
    errs = pu.measure(w, bad, ref)
    with pytest.raises(AssertionError):
        pu.gate("x", errs, 1e-4)
    key2 = ("grad_inf", 0, "linear0.W")
    worst, ill = pu.gate("x", errs, 1e-4, sens={key: (errs[key][0], 0.0), key2: (errs[key2][0], 0.0)})
    assert sorted(i[0] for i in ill) == sorted([key, key2])


def test_argmax_comparison_skips_only_unresolvable_rows():
    w = wl.config1(B=8, D=24, hidden=12)
    ref = pu.run_oracle(w, 1)
    logits = [np.array([[0.0, 1.0, 0.5]] * 8, dtype=np.float32)] * 2
    pred = [np.ones(8, dtype=np.int32)] * 2
    assert pu.compare_pred(w, pred, logits, pred, 1e-4) == (16, 0)
    wrong = [np.zeros(8, dtype=np.int32)] * 2
    with pytest.raises(AssertionError):
        pu.compare_pred(w, wrong, logits, pred, 1e-4)
    tie = [np.array([[1.0, 1.0, 0.5]] * 8, dtype=np.float32)] * 2
    assert pu.compare_pred(w, wrong, tie, pred, 1e-4) == (0, 16)


def test_oracle_sensitivity_is_small_for_a_well_conditioned_pack():
    w = wl.config2(B=32, D=64, hidden=(32, 32), K=2, steps=2)
    base = pu.run_oracle(w, 2, mode="rounded")
    sens = pu.oracle_sensitivity(w, 2, base, trials=1)
    assert max(v[0] for v in sens.values()) < 5e-3
