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


def test_ill_conditioned_items_are_reported_not_hidden_and_only_where_allowed():
    w = wl.config1(B=8, D=24, hidden=12)
    ref = pu.run_oracle(w, 1)
    bad = _as_gpu(ref)
    bad["grads"][0][3] *= 1.05                       # one entry of one tensor, as a flipped unit would move it
    errs = pu.measure(w, bad, ref)
    k2, kinf = ("grad_l2", 0, "linear0.W"), ("grad_inf", 0, "linear0.W")
    assert errs[kinf][0] > 1e-4
    with pytest.raises(AssertionError):                  # nothing vouches for the item
        pu.gate("x", errs, 1e-4)
    big = {k2: (1.0, 0.0), kinf: (1.0, 0.0)}
    if errs[k2][0] > 1e-4:
        # a 2-norm at step 1 gets no allowance, however sensitive the oracle says it is
        with pytest.raises(AssertionError):
            pu.gate("x", errs, 1e-4, sens=big)
        errs[k2] = (0.0, 0.0)
    called = []
    worst, took, n = pu.gate("x", errs, 1e-4, sens=lambda: called.append(1) or big, max_share=1.0)
    assert [t[0] for t in took] == [kinf] and called == [1]
    with pytest.raises(AssertionError):                  # sensitivity too small to explain the error
        pu.gate("x", errs, 1e-4, sens={kinf: (1e-6, 0.0)}, max_share=1.0)
    with pytest.raises(AssertionError):                  # explained, but beyond tol + 4 x sensitivity
        pu.gate("x", errs, 1e-4, sens={kinf: (errs[kinf][0] / 5, 0.0)}, max_share=1.0)
    with pytest.raises(AssertionError):                  # too large a share of the items needs the allowance
        pu.gate("x", errs, 1e-4, sens=big, max_share=0.01)
    # the sensitivity is not even computed when everything is within tolerance
    good = pu.measure(w, _as_gpu(ref), ref)
    pu.gate("x", good, 1e-4, sens=lambda: 1 / 0)


def test_multi_step_displacement_may_take_the_allowance_a_first_step_one_may_not():
    w = wl.config1(B=8, D=24, hidden=12)
    ref = pu.run_oracle(w, 2)
    bad = _as_gpu(ref)
    bad["blobs"][0] = (w.weights[0] + (ref["blobs"][0] - w.weights[0]) * 1.01).astype(np.float32)
    errs = {k: v for k, v in pu.measure(w, bad, ref).items() if k[0] == "disp_l2"}
    sens = {k: (1.0, 0.0) for k in errs}
    pu.gate("x", errs, 1e-4, sens=sens, steps=2, max_share=1.0)
    with pytest.raises(AssertionError):
        pu.gate("x", errs, 1e-4, sens=sens, steps=1, max_share=1.0)


def test_argmax_comparison_skips_only_unresolvable_rows():
    w = wl.config1(B=8, D=24, hidden=12)
    base = np.array([[0.0, 1.0, 0.5]] * 8)
    ref_logits = [base.copy(), base.copy()]
    logits = [(base + 1e-3).astype(np.float32)] * 2        # measured logit error 1e-3: gap 0.5 is resolvable
    pred = [np.ones(8, dtype=np.int32)] * 2
    n, skipped, err = pu.compare_pred(w, pred, logits, pred, ref_logits)
    assert (n, skipped) == (16, 0) and abs(err - 1e-3) < 1e-6
    wrong = [np.zeros(8, dtype=np.int32)] * 2
    with pytest.raises(AssertionError):
        pu.compare_pred(w, wrong, logits, pred, ref_logits)
    # rows whose oracle gap is below four times the measured error are skipped, the others still compared
    close = base.copy()
    close[:2] = [0.998, 1.0, 0.5]
    dev = close.copy()
    dev[:2] = [1.0, 0.9985, 0.5]                           # the device orders the near-tie the other way
    dev_pred = np.argmax(dev, axis=1).astype(np.int32)
    ref_pred = np.argmax(close, axis=1).astype(np.int32)
    n, skipped, err = pu.compare_pred(w, [dev_pred] * 2, [dev.astype(np.float32)] * 2, [ref_pred] * 2, [close] * 2,
                                      max_skipped_share=0.5)
    assert (n, skipped) == (12, 4)
    with pytest.raises(AssertionError):                    # too many rows skipped
        pu.compare_pred(w, [dev_pred] * 2, [dev.astype(np.float32)] * 2, [ref_pred] * 2, [close] * 2, max_skipped_share=0.1)
    with pytest.raises(AssertionError):                    # the device's argmax must be that of its own logits
        pu.compare_pred(w, [ref_pred] * 2, [dev.astype(np.float32)] * 2, [ref_pred] * 2, [close] * 2, max_skipped_share=0.5)


def test_oracle_sensitivity_is_small_for_a_well_conditioned_pack():
    w = wl.config2(B=32, D=64, hidden=(32, 32), K=2, steps=2)
    base = pu.run_oracle(w, 2, mode="rounded")
    sens = pu.oracle_sensitivity(w, 2, base, trials=1)
    assert max(v[0] for v in sens.values()) < 2e-3
