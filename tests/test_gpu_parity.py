"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Tolerances: 1e-4 (fp32 packs) and 2e-2 (bf16 packs) maximum relative error; labels,
argmax and everything integer must agree exactly."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pack_oracle as po
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

F32_TOL, BF16_TOL = pu.TOL[wl.F32], pu.TOL[wl.BF16]


def _member(w, k):
    """Member k of workload `w` as a workload of its own (same shared batch, its own slice of it)."""
    solo = wl.PackWorkload(w.name, w.dtype, w.B, w.in_shape, [w.models[k]], [w.batch[k]], [w.weights[k]],
                           w.lr[k:k + 1], w.x, w.labels, w.steps, w.n_classes)
    if w.meta.get("optimizers"):
        solo.meta["optimizers"] = [w.meta["optimizers"][k]]
    return solo


def _same_bits(a, b, what=("blobs", "loss")):
    for key in what:
        if key == "loss":
            assert np.array_equal(a["loss"], b["loss"])
        else:
            for x, y in zip(a[key], b[key]):
                assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), key


def _check_production_form(w, steps, gpu):
    """The gradient-storing form of the fused weight-gradient + update kernels is what the comparisons
    with the oracle read their gradients from; the form a caller gets by default stores no gradient.
    Both must leave the same weights and losses, bit for bit."""
    _same_bits(pu.run_gpu(w, steps, keep_first_grads=False), gpu)


def _small(w):
    """A reduced test case: fewer than 64 rows per member, where one flipped unit shows in a 2-norm."""
    return max(w.batch) < 64


def _check_f32(w, steps=None, trials=2, production_form=False):
    """fp32 packs against the float64 oracle at 1e-4: every loss, the step-1 gradients and the
    displacement of every tensor in the 2-norm and the infinity norm, the raw weights.  Single entries
    (infinity norms) and several-step displacements that exceed it must be explained by the oracle's
    own sensitivity to fp32-sized accumulation noise (parity_util.gate), and only a bounded share of
    them may need that."""
    steps = w.steps if steps is None else steps
    gpu = pu.run_gpu(w, steps)
    ref = pu.run_oracle(w, steps)
    worst = pu.compare(w, gpu, ref, F32_TOL, sens=lambda: pu.oracle_sensitivity(w, steps, ref, mode="exact", trials=trials),
                       small_case=_small(w))
    n, skipped, lerr = pu.compare_pred(w, gpu["pred_first"], gpu["logits"], ref["pred"][0], ref["logits"][0])
    if production_form:
        _check_production_form(w, steps, gpu)
    print(f"\n{w.name}: worst {worst}; argmax rows compared {n}, unresolvable {skipped} (largest logit difference {lerr:.1e}); "
          f"launches {gpu['launches']}")
    return gpu, ref


def _check_bf16(w, steps=None, trials=2, production_form=False):
    """bf16 packs (bf16 inputs/weights, fp32 accumulate, fp32 master).  Three references:
    - step 1 against the float64 oracle (the weights are bf16-representable, so the only
      difference is the rounding of stored activations): loss within 2e-2;
    - every step against the oracle that rounds where the device rounds: loss, step-1
      gradients, displacement and weights within 2e-2, gated as for fp32 packs (parity_util.gate);
    - every step against the oracle that only rounds the per-step weight copy (the precision
      the configuration itself fixes): every loss, and the 2-norm of every tensor's displacement, no
      farther from it than the rounding oracle itself lies plus 2e-2, no item excluded."""
    steps = w.steps if steps is None else steps
    gpu = pu.run_gpu(w, steps)
    exact = pu.run_oracle(w, 1, mode="exact")
    weights = pu.run_oracle(w, steps, mode="weights")
    rounded = pu.run_oracle(w, steps, mode="rounded")
    first = {"loss": gpu["loss"][:1], "blobs": gpu["blobs"], "grads": None}
    w0 = pu.compare(w, first, exact, BF16_TOL, what=("loss",), label="exact step 1: ")
    w2 = pu.compare(w, gpu, rounded, BF16_TOL, what=("loss", "grads", "disp", "weights"), label="rounded: ",
                    sens=lambda: pu.oracle_sensitivity(w, steps, rounded, trials=trials), small_case=_small(w))
    vs_weights = _check_against_weight_rounding(w, gpu, weights, rounded, w2)
    n, skipped, lerr = pu.compare_pred(w, gpu["pred_first"], gpu["logits"], rounded["pred"][0], rounded["logits"][0])
    if production_form:
        _check_production_form(w, steps, gpu)
    print(f"\n{w.name}: step-1 loss vs float64 {w0['loss']:.2e}; vs rounding oracle {w2}; "
          f"vs weight-rounding oracle (device error, and how far the rounding oracle itself lies from it) {vs_weights}; "
          f"argmax rows {n}, unresolvable {skipped} (largest logit difference {lerr:.1e}); launches {gpu['launches']}")
    return gpu, weights, rounded


def _check_against_weight_rounding(w, gpu, weights, rounded, vs_rounded=None):
    """Loss at every step and the 2-norm displacement of every tensor against the oracle that rounds
    only the per-step weight copy (the precision the configuration itself fixes).  Storing activations
    and gradients in bf16 moves the oracle itself away from that reference (`own`: how far its mode
    "rounded" lies from its mode "weights"); the device may lie no farther from it than that plus the
    tolerance (plus, for an item that needed the ill-conditioning allowance in the comparison with the
    rounding oracle, `vs_rounded`, that same allowance: the bound is the triangle inequality through the
    rounding oracle).  No item is excluded.  Returns the worst device error, the worst `own`, for losses
    and for displacements."""
    worst = {"loss": 0.0, "loss_own": 0.0, "disp_l2": 0.0, "disp_l2_own": 0.0}
    extra = {(key[1], key[2]): 4 * sens for key, sens, _ in (vs_rounded or {}).get("ill_conditioned", []) if key[0] == "disp_l2"}
    extra_loss = {}
    for key, sens, _ in (vs_rounded or {}).get("ill_conditioned", []):
        if key[0] == "loss":
            extra_loss[key[1]] = max(extra_loss.get(key[1], 0.0), 4 * sens)
    for k in range(w.K):
        # (once two trajectories have drifted apart they may cross again: the largest distance so far counts)
        own = np.maximum.accumulate(np.abs(weights["loss"][:, k] - rounded["loss"][:, k]) / np.abs(weights["loss"][:, k]))
        err = np.abs(gpu["loss"][:, k] - weights["loss"][:, k]) / np.abs(weights["loss"][:, k])
        assert np.all(err <= own + BF16_TOL + extra_loss.get(k, 0.0)), f"{w.name} member {k}: loss vs weight-rounding oracle {err}, the oracles differ by {own}"
        worst["loss"], worst["loss_own"] = max(worst["loss"], float(err.max())), max(worst["loss_own"], float(own.max()))
        if float(w.lr[k]) == 0.0:
            continue
        w0 = w.weights[k].astype(np.float64)
        for name, s in pu.tensor_slices(w.models[k], w.in_shape):
            d_ref, d_rnd = weights["blobs"][k][s] - w0[s], rounded["blobs"][k][s] - w0[s]
            d_gpu = gpu["blobs"][k][s].astype(np.float64) - w0[s]
            own, e = pu.rel_l2(d_rnd, d_ref), pu.rel_l2(d_gpu, d_ref)
            assert e <= own + BF16_TOL + extra.get((k, name), 0.0), f"{w.name} member {k} {name}: displacement vs weight-rounding oracle {e}, the oracles differ by {own}"
            worst["disp_l2"], worst["disp_l2_own"] = max(worst["disp_l2"], e), max(worst["disp_l2_own"], own)
    return {key: float(f"{v:.3g}") for key, v in worst.items()}


# ------------------------------------------------------------------ MLPs, fp32
def test_c1_two_mlps_fp32_full_size():
    _check_f32(wl.config1())


def test_mlp_fp32_ragged_shapes_and_batch_slices():
    models = [wl.mlp([50], 7), wl.mlp([33, 130], 7), wl.mlp([129, 5, 64], 7), [("linear", 7)]]
    w = wl.custom("ragged_f32", 5, wl.F32, 19, (1, 1, 37), models, batch=[19, 7, 1, 13], n_classes=7, steps=3)
    _check_f32(w)


def test_mlp_fp32_spans_several_tiles():
    models = [wl.mlp([300, 260], 10), wl.mlp([140], 10)]
    w = wl.custom("tiles_f32", 6, wl.F32, 300, (1, 1, 200), models, batch=[300, 150], n_classes=10, steps=2,
                  lr=[0.05, 0.02])
    _check_f32(w)


# ------------------------------------------------------------------ MLPs, bf16
def test_c2_reduced_bf16():
    _check_bf16(wl.config2(B=64, D=256, hidden=(128, 136), K=3, steps=3))


@pytest.mark.parametrize("K", [1, 3, 4, 16])
def test_identical_members_whose_weight_gradient_tiles_are_dealt_to_the_xcds_by_member(K, monkeypatch):
    # K = 4: each member cut into two parts (column strips 3 and 2 wide); K = 16: two members per XCD;
    # K = 3: falls back to the rotating deal.  Both deals must give the same bits.
    w = wl.config2(B=160, D=384, hidden=(640, 272), K=K, steps=2)
    _check_bf16(w, trials=1)
    by_member = pu.run_gpu(w, steps=2, keep_first_grads=False)
    monkeypatch.setenv("PACK_XCD_ROTATE", "1")
    rotating = pu.run_gpu(w, steps=2, keep_first_grads=False)
    for a, b in zip(by_member["blobs"], rotating["blobs"]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_c2_eight_mlps_bf16_full_size():
    _check_bf16(wl.config2(), trials=1, production_form=True)


def test_c4_reduced_heterogeneous_bf16():
    _check_bf16(wl.config4(K=6, B=32, D=96, width_choices=(8, 16, 40, 64), steps=3))


@pytest.mark.parametrize("n_classes", [10, 100])
def test_c4_heterogeneous_bf16_full_size(n_classes):
    _check_bf16(wl.config4(n_classes=n_classes), trials=1, production_form=True)


# ------------------------------------------------------------------ CNNs
def test_c3_reduced_fp32():
    _check_f32(wl.config3(K=2, B=5, size=10, widths=(8, 12, 20), steps=3))


def test_c3_reduced_fp32_odd_sizes():
    _check_f32(wl.config3(K=2, B=3, size=7, widths=(5, 9, 6), steps=2))


@pytest.mark.timeout(900)
def test_c3_four_cnns_fp32_full_size_all_five_steps():
    _check_f32(wl.config3(), trials=1, production_form=True)


def test_c5_reduced_fp32_and_bf16():
    _check_f32(wl.config5(K=2, B=3, size=12, widths=(8, 16, 24, 32), n_classes=10, steps=2, dtype=wl.F32))
    _check_bf16(wl.config5(K=2, B=4, size=16, widths=(8, 16, 32, 64), n_classes=10, steps=2))


@pytest.mark.parametrize("make", [
    lambda: wl.config5(K=2, B=8, size=16, steps=2),                                   # bf16, 128 x 64 and 128 x 128 tiles
    lambda: wl.config3(K=2, B=16, size=16, widths=(32, 64, 128), steps=2),            # fp32
    lambda: wl.config2(B=256, D=384, hidden=(64, 192), K=3, steps=2),                 # dense layers, bf16
])
def test_lean_form_of_forward_and_input_gradient_tiles_gives_the_same_bits(make, monkeypatch):
    # the occupancy-bound form of the 128 x 64 kernels multiplies the same chunks in the same order:
    # forced on for every reduction length and tile count, it must reproduce the regular form exactly
    w = make()
    monkeypatch.setenv("PACK_MIN_TILES", "1")       # small layers keep the 128-row tiles they would get in a large pack
    monkeypatch.setenv("PACK_LEAN64_CHUNKS", "0")
    regular = pu.run_gpu(w, steps=2)
    monkeypatch.setenv("PACK_LEAN64_CHUNKS", "100000")
    lean = pu.run_gpu(w, steps=2)
    assert not any(t == (128, 64, True) for t in regular["tiles"])
    assert any(t == (128, 64, True) for t in lean["tiles"])
    for a, b in zip(regular["blobs"], lean["blobs"]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for a, b in zip(regular["logits"], lean["logits"]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for a, b in zip(regular["grads"], lean["grads"]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("make", [
    lambda: wl.config5(K=2, B=8, size=16, steps=2),                                   # bf16: 16 and 8 pixel rows, both strides; 4 pixel rows stay on the staged tiles
    lambda: wl.config5(K=2, B=2, size=64, widths=(64, 128), n_classes=10, steps=2),   # bf16: 64 and 32 pixel rows (one and two rows per chunk)
    lambda: wl.config3(K=2, B=16, size=32, widths=(32, 64, 128), steps=2),            # fp32: 32 input channels per tile; stride 2, 16 pixel rows
    lambda: wl.config5(K=1, B=4, size=32, widths=(64, 64), n_classes=10, steps=2, dtype=wl.F32),   # fp32, stride 1 and 2
    lambda: wl.config3(K=2, B=4, size=32, widths=(32, 64, 64), steps=2, dtype=wl.BF16),            # bf16, 32 input channels per tile
])
def test_halo_form_of_the_convolution_weight_gradient_gives_the_same_bits_as_the_staged_tiles(make, monkeypatch):
    # all nine taps of a block of channel pairs in one workgroup, the input staged once per chunk of pixels:
    # same chunks, same order inside them, same splits, so the same bits as the form it replaces
    w = make()
    halo = pu.run_gpu(w, steps=2)
    assert any(t[:2] in ((64, 576), (64, 288)) for t in halo["tiles"])
    monkeypatch.setenv("PACK_NO_HALO_DW", "1")
    staged = pu.run_gpu(w, steps=2)
    assert not any(t[:2] in ((64, 576), (64, 288)) for t in staged["tiles"])
    for key in ("grads", "blobs"):
        for a, b in zip(halo[key], staged[key]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), key
    assert np.array_equal(halo["loss"], staged["loss"])


@pytest.mark.parametrize("make,one_block", [
    (lambda: wl.config5(K=2, B=4, size=64, widths=(64, 64), n_classes=10, steps=2), True),     # bf16, 64 channels: one block; 64 and 32 pixel rows
    (lambda: wl.config3(K=2, B=16, size=32, widths=(32, 32, 64), steps=2), True),              # fp32, 32 channels: one block; 32-column input gradient
    (lambda: wl.config5(K=2, B=16, size=32, steps=2), False),                                  # bf16, up to 512 channels; 32 to 4 pixel rows (whole images per tile)
    (lambda: wl.config5(K=1, B=8, size=32, widths=(64, 128), n_classes=10, steps=2, dtype=wl.F32), False),   # fp32, several blocks
])
def test_halo_form_of_stride_1_forward_and_input_gradient_against_the_staged_tiles(make, one_block, monkeypatch):
    # the pixels a tile's nine taps reach staged once per block of channels.  With one channel block the
    # reduction order is that of the staged-tile form (the same bits); with several it runs block by block
    # instead of tap by tap: the same sums in another order
    w = make()
    halo = pu.run_gpu(w, steps=2)
    assert any(t[:2] in ((256, 64), (256, 32)) for t in halo["tiles"]), halo["tiles"]
    monkeypatch.setenv("PACK_NO_HALO_ROWS", "1")
    staged = pu.run_gpu(w, steps=2)
    assert not any(t[:2] in ((256, 64), (256, 32)) for t in staged["tiles"])
    for key in ("grads", "blobs", "logits"):
        for a, b in zip(halo[key], staged[key]):
            if one_block:
                assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), key
            else:
                scale = float(np.max(np.abs(b))) + 1e-30
                tol = (BF16_TOL if w.dtype == wl.BF16 else F32_TOL)
                assert float(np.max(np.abs(a.astype(np.float64) - b.astype(np.float64)))) <= tol * scale, key
    if one_block:
        assert np.array_equal(halo["loss"], staged["loss"])


@pytest.mark.parametrize("make", [
    lambda: wl.config5(K=2, B=8, size=32, steps=2),                                    # bf16: residual blocks, both strides, parity classes
    lambda: wl.config3(K=2, B=16, size=32, widths=(32, 64, 128), steps=2),             # fp32 convolutions
    lambda: wl.config2(B=256, D=384, hidden=(128, 192), K=3, steps=2),                 # dense layers, bf16
    lambda: wl.config4(K=4, B=128, D=256, steps=2),                                    # ragged dense layers and batches
])
def test_the_tail_of_whole_plain_tiles_gives_the_same_bits_as_the_general_tail(make, monkeypatch):
    # whole tiles of the plain cases take a tail with strength-reduced addresses and hoisted flags; which tiles do
    # depends on the tile shape, which depends on the pack, so it must not change a single bit
    w = make()
    fast = pu.run_gpu(w, steps=2)
    monkeypatch.setenv("PACK_GENERAL_TAIL", "1")
    general = pu.run_gpu(w, steps=2)
    for key in ("grads", "blobs", "logits"):
        for a, b in zip(fast[key], general[key]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), key
    assert np.array_equal(fast["loss"], general["loss"])


def test_c5_resnet_style_bf16_full_width_reduced_images():
    _check_bf16(wl.config5(K=2, B=8, size=16, steps=2))


def test_c5_resnet_style_full_width_32px_bf16_and_fp32():
    # power-of-two maps of 32, 16, 8 and 4 pixels at the full channel widths: the aligned
    # (vector gather) forms of all three convolution products, both element types
    _check_bf16(wl.config5(K=2, B=4, size=32, steps=1), trials=1)
    _check_f32(wl.config5(K=1, B=4, size=32, steps=1, dtype=wl.F32), trials=1)


@pytest.mark.timeout(1500)
def test_c5_four_resnet_style_cnns_bf16_full_size():
    """The largest configuration at its real size (64 x 64 images, batch 64, K = 4), one step.  One oracle
    step of one member takes minutes of CPU time, so ONE member is compared with the oracle (with the
    device's rounding points: loss, every gradient, every displacement; with only the weight copy
    rounded: loss and 2-norm displacements) and the others by what Section 2.2 guarantees: each must
    equal, bit for bit, the same member trained alone, which is itself checked for member 0.  Then the
    default form of the kernels (no gradient stored) must reproduce the gradient-storing run's bits."""
    w = wl.config5()
    gpu = pu.run_gpu(w, 1)
    k = 0
    solo = _member(w, k)
    rounded = pu.run_oracle(solo, 1, mode="rounded")
    one = {key: ([gpu[key][k]] if isinstance(gpu[key], list) else gpu[key]) for key in ("grads", "logits", "pred_first", "blobs")}
    one["loss"] = gpu["loss"][:, k:k + 1]
    w2 = pu.compare(solo, one, rounded, BF16_TOL, label="rounded: ",
                    sens=lambda: pu.oracle_sensitivity(solo, 1, rounded, trials=1))
    weights = pu.run_oracle(solo, 1, mode="weights")
    vs_weights = _check_against_weight_rounding(solo, one, weights, rounded, w2)
    n, skipped, lerr = pu.compare_pred(solo, one["pred_first"], one["logits"], rounded["pred"][0], rounded["logits"][0])
    for j in range(w.K):
        alone = pu.run_gpu(_member(w, j), 1)
        assert np.array_equal(alone["blobs"][0].view(np.uint32), gpu["blobs"][j].view(np.uint32)), j
        assert np.array_equal(alone["grads"][0].view(np.uint32), gpu["grads"][j].view(np.uint32)), j
        assert np.array_equal(alone["loss"][:, 0], gpu["loss"][:, j]), j
    _check_production_form(w, 1, gpu)
    print(f"\nc5 full size: member {k} vs rounding oracle {w2}; vs weight-rounding oracle {vs_weights}; "
          f"argmax rows {n}, unresolvable {skipped} (largest logit difference {lerr:.1e}); launches {gpu['launches']}")


# ------------------------------------------------------------------ the paper's invariants on the device
def _blobs_equal(a, b):
    return all(np.array_equal(x, y) for x, y in zip(a, b))


def test_singleton_pack_and_run_to_run_determinism():
    w = wl.config2(B=32, D=128, hidden=(64, 64), K=1, steps=3)
    a = pu.run_gpu(w)
    b = pu.run_gpu(w)
    assert _blobs_equal(a["blobs"], b["blobs"]) and np.array_equal(a["loss"], b["loss"])
    _check_bf16(w)


def test_member_result_does_not_depend_on_the_rest_of_the_pack():
    # Section 2.2: a member trains as if alone -> bit-identical whether packed with others or not,
    # whatever the others' learning rates, and wherever it sits in the pack.
    w = wl.config4(K=5, B=64, D=160, width_choices=(24, 64, 136), steps=3)
    full = pu.run_gpu(w)
    for k in (0, 3):
        solo = wl.PackWorkload(w.name, w.dtype, w.B, w.in_shape, [w.models[k]], [w.batch[k]], [w.weights[k]],
                               w.lr[k:k + 1], w.x, w.labels, w.steps, w.n_classes)
        one = pu.run_gpu(solo)
        assert np.array_equal(one["blobs"][0], full["blobs"][k])
        assert np.array_equal(one["loss"][:, 0], full["loss"][:, k])
    lr2 = w.lr.copy()
    lr2[1] *= 3.0
    other = pu.run_gpu(w, lr=lr2)
    for k in (0, 2, 3, 4):
        assert np.array_equal(other["blobs"][k], full["blobs"][k])
    assert not np.array_equal(other["blobs"][1], full["blobs"][1])
    perm = [3, 1, 4, 0, 2]
    wp = wl.PackWorkload(w.name, w.dtype, w.B, w.in_shape, [w.models[i] for i in perm], [w.batch[i] for i in perm],
                         [w.weights[i] for i in perm], w.lr[perm], w.x, w.labels, w.steps, w.n_classes)
    shuffled = pu.run_gpu(wp)
    for j, i in enumerate(perm):
        assert np.array_equal(shuffled["blobs"][j], full["blobs"][i])
        assert np.array_equal(shuffled["pred"][j], full["pred"][i])


def test_rows_beyond_a_members_batch_are_never_read():
    w = wl.config4(K=4, B=32, D=64, width_choices=(16, 32), steps=2, dtype=wl.F32)
    w.batch = [32, 8, 16, 5]
    base = pu.run_gpu(w)
    x2 = w.x.copy()
    x2[16:] = 7.0
    lab2 = w.labels.copy()
    lab2[16:] = (lab2[16:] + 1) % w.n_classes
    w2 = wl.PackWorkload(w.name, w.dtype, w.B, w.in_shape, w.models, w.batch, w.weights, w.lr, x2, lab2, w.steps, w.n_classes)
    moved = pu.run_gpu(w2)
    for k in (1, 2, 3):
        assert np.array_equal(base["blobs"][k], moved["blobs"][k])
    assert not np.array_equal(base["blobs"][0], moved["blobs"][0])


def test_zero_learning_rate_leaves_weights_bit_identical():
    w = wl.config3(K=2, B=4, size=8, widths=(8, 8, 8), steps=2)
    out = pu.run_gpu(w, lr=[0.0, 0.01])
    assert np.array_equal(out["blobs"][0], w.weights[0])
    assert not np.array_equal(out["blobs"][1], w.weights[1])


def test_exact_ties_in_the_logits_and_label_column():
    # A linear-only member with zero weights: its logits are exactly its bias for every row, so
    # ties are exact; argmax must return the lowest index and the loss must use column y.
    C, D, B = 6, 16, 9
    bias = np.array([1.0, 3.0, 3.0, 2.0, 3.0, -1.0], dtype=np.float32)
    blob = np.concatenate([np.zeros(C * D, dtype=np.float32), bias])
    for dtype in (wl.F32, wl.BF16):
        w = wl.custom("ties", 9, dtype, B, (1, 1, D), [[("linear", C)]], n_classes=C, lr=[0.0])
        w.weights = [blob]
        gpu = pu.run_gpu(w)
        ref = pu.run_oracle(w)
        assert np.array_equal(gpu["pred"][0], np.ones(B, dtype=np.int32))
        assert np.array_equal(gpu["pred"][0], ref["pred"][0][0])
        assert np.array_equal(gpu["logits"][0], np.tile(bias, (B, 1)))
        assert abs(gpu["loss"][0, 0] - ref["loss"][0, 0]) <= 1e-6 * ref["loss"][0, 0]
        tol = 1e-6 if dtype == wl.F32 else 2.0 ** -8
        assert pu.rel_inf(gpu["grads"][0].astype(np.float64), ref["grads"][0][0]) <= tol


def test_out_of_range_label_is_reported_and_never_indexes_memory():
    from paper_2002_02885_amd import binding
    w = wl.config1(B=8, D=16, hidden=8)
    lab = w.labels.copy()
    lab[3] = 10
    lab[5] = -1
    pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
    try:
        for k in range(w.K):
            pk.write_weights(k, w.weights[k])
        x = torch.from_numpy(w.x).cuda()
        y = torch.from_numpy(lab).cuda()
        pk.step(x.data_ptr(), y.data_ptr(), w.lr)
        loss = pk.read_loss(allow_label_error=True)
        assert pk.last_status == binding.PACK_ELABEL and np.all(np.isfinite(loss))
        ok = np.ones(8, dtype=bool)
        ok[[3, 5]] = False
        # rows with a bad label contribute nothing: same loss sum as the oracle on the good rows
        from oracle import pack_oracle as po
        for k in range(w.K):
            net = po.Model(w.models[k], w.in_shape, w.weights[k].astype(np.float64))
            l6, _, _ = net.loss_and_grads(w.x[ok].astype(np.float64), w.labels[ok])
            assert abs(loss[k] - l6 * 6 / 8) <= 1e-4 * abs(l6)
        y2 = torch.from_numpy(w.labels).cuda()
        pk.step(x.data_ptr(), y2.data_ptr(), w.lr)
        pk.read_loss()
        assert pk.last_status == binding.PACK_OK
    finally:
        pk.destroy()


def test_seeded_initialisation_is_reproducible_and_bounded():
    from paper_2002_02885_amd import binding
    models = [wl.small_cnn((8, 8, 8), 10)]
    a = binding.Pack(2, (8, 8, 3), "f32", models, seed=42)
    b = binding.Pack(2, (8, 8, 3), "f32", models, seed=42)
    c = binding.Pack(2, (8, 8, 3), "f32", models, seed=43)
    wa, wb, wc = a.read_weights(0), b.read_weights(0), c.read_weights(0)
    a.destroy(); b.destroy(); c.destroy()
    assert np.array_equal(wa, wb) and not np.array_equal(wa, wc)
    off = 0
    for kind, ws, bs, fan_in in wl.param_shapes(models[0], (8, 8, 3)):
        nw, nb = int(np.prod(ws)), int(np.prod(bs))
        W, bb = wa[off:off + nw], wa[off + nw:off + nw + nb]
        off += nw + nb
        assert np.max(np.abs(W)) <= np.sqrt(6.0 / fan_in) and np.max(np.abs(bb)) <= 1 / np.sqrt(fan_in)
        assert np.max(np.abs(W)) > 0.8 * np.sqrt(6.0 / fan_in) and abs(W.mean()) < 0.2 * np.sqrt(6.0 / fan_in)


# ------------------------------------------------------------------ the rest of the paper's search space (Table 3)
ADAM = {"kind": "adam", "beta1": 0.9, "beta2": 0.999, "eps": 1e-8}
MOMENTUM = {"kind": "momentum", "mu": 0.9}
ADAGRAD = {"kind": "adagrad", "acc0": 0.1}
SGD = {"kind": "sgd"}


def _act_mlp(widths, act, C=10):
    layers = []
    for h in widths:
        layers += [("linear", h), (act,)]
    return layers + [("linear", C)]


def _check_opt_state(w, gpu, ref, tol):
    """Optimiser state after the last step against the oracle's, per member and state array,
    relative to the largest entry (Adam's second moment spans many orders of magnitude)."""
    for k, opt in enumerate(w.meta["optimizers"]):
        for slot, (state, steps) in enumerate(gpu["opt_state"][k]):
            want = ref["nets"][k].opt_state_blob(slot)
            assert steps == ref["nets"][k].t
            err = np.max(np.abs(state - want)) / max(np.max(np.abs(want)), 1e-300)
            assert err <= tol, f"{w.name} member {k} {opt['kind']} state {slot}: {err}"


def test_activations_and_optimisers_mlp_fp32():
    """One pack whose members differ in activation AND optimiser (Table 2 'Optimizer: Different',
    Table 3), ragged widths and batch slices, several steps."""
    models = [_act_mlp([96, 40], "tanh"), _act_mlp([130], "sigmoid"), _act_mlp([64, 64, 24], "leaky_relu"),
              _act_mlp([72], "relu"), _act_mlp([50, 30], "tanh")]
    w = wl.custom("acts_opts_f32", 41, wl.F32, 48, (1, 1, 200), models, batch=[48, 40, 48, 17, 48],
                  lr=lambda r: np.array([1e-3, 5e-2, 2e-2, 5e-2, 1e-2]), steps=4)
    w.meta["optimizers"] = [ADAM, MOMENTUM, ADAGRAD, SGD, {"kind": "adam", "beta1": 0.8, "beta2": 0.95, "eps": 1e-6}]
    gpu, ref = _check_f32(w)
    _check_opt_state(w, gpu, ref, F32_TOL)


def test_activations_and_optimisers_cnn_fp32():
    cnn = lambda a, b: [("conv3x3", 8, 1), (a,), ("conv3x3", 16, 2), (b,), ("gap",), ("linear", 10)]
    models = [cnn("tanh", "leaky_relu"), cnn("sigmoid", "relu"), cnn("leaky_relu", "tanh")]
    w = wl.custom("acts_opts_cnn_f32", 42, wl.F32, 12, (10, 10, 3), models, lr=lambda r: np.array([2e-3, 3e-2, 3e-2]),
                  pixel="uniform", steps=3)
    w.meta["optimizers"] = [ADAM, ADAGRAD, MOMENTUM]
    gpu, ref = _check_f32(w)
    _check_opt_state(w, gpu, ref, F32_TOL)


def test_activations_and_optimisers_bf16():
    models = [_act_mlp([128, 64], "tanh"), _act_mlp([128], "sigmoid"), _act_mlp([64, 64], "leaky_relu"), _act_mlp([128], "relu")]
    w = wl.custom("acts_opts_bf16", 43, wl.BF16, 64, (1, 1, 256), models, lr=lambda r: np.array([1e-3, 2e-2, 2e-2, 2e-2]), steps=4)
    w.meta["optimizers"] = [ADAM, MOMENTUM, ADAGRAD, MOMENTUM]
    gpu, weights, rounded = _check_bf16(w)
    _check_opt_state(w, gpu, rounded, BF16_TOL)


def test_optimiser_checkpoint_round_trip_continues_the_same_trajectory():
    """free's checkpoint carries the optimiser state (Section 2.2): train 2 steps, read weights and
    state, load them into a fresh pack, train 2 more; bit-identical to 4 uninterrupted steps."""
    from paper_2002_02885_amd import binding
    models = [_act_mlp([64], "tanh"), _act_mlp([32, 32], "relu")]
    w = wl.custom("ckpt", 44, wl.F32, 16, (1, 1, 40), models, lr=lambda r: np.array([1e-2, 1e-2]), steps=4)
    opts = [ADAM, MOMENTUM]
    x_dev, y_dev = pu.device_inputs(w)

    def fresh():
        pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
        for k in range(w.K):
            pk.write_weights(k, w.weights[k])
            pk.set_optimizer(k, opts[k])
        return pk

    a = fresh()
    for _ in range(4):
        a.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
    want = [a.read_weights(k) for k in range(w.K)]
    a.destroy()
    b = fresh()
    for _ in range(2):
        b.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
    ckpt = [(b.read_weights(k), [b.read_opt_state(k, s) for s in range(2 if opts[k]["kind"] == "adam" else 1)]) for k in range(w.K)]
    b.destroy()
    c = fresh()
    for k, (blob, states) in enumerate(ckpt):
        c.write_weights(k, blob)
        for s, (arr, steps) in enumerate(states):
            assert steps == 2
            c.write_opt_state(k, s, arr, steps)
    for _ in range(2):
        c.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
    got = [c.read_weights(k) for k in range(w.K)]
    c.destroy()
    for k in range(w.K):
        assert np.array_equal(got[k], want[k])


def test_optimiser_argument_errors():
    from paper_2002_02885_amd import binding
    pk = binding.Pack(4, (1, 1, 8), wl.F32, [[("linear", 3)]], [4])
    try:
        for bad in ({"kind": "momentum", "mu": 1.0}, {"kind": "adagrad", "acc0": 0.0}, {"kind": "adam", "eps": 0.0},
                    {"kind": "adam", "beta2": 1.5}):
            with pytest.raises(binding.PackError) as e:
                pk.set_optimizer(0, bad)
            assert e.value.status == binding.PACK_EINVAL
        with pytest.raises(binding.PackError):
            pk.read_opt_state(0, 0)            # plain SGD has no state
        pk.set_optimizer(0, MOMENTUM)
        with pytest.raises(binding.PackError):
            pk.read_opt_state(0, 1)            # momentum has one state array
        assert pk.read_opt_state(0, 0)[1] == 0
    finally:
        pk.destroy()


def test_update_in_the_gradient_kernels_equals_the_separate_update_bit_for_bit(monkeypatch):
    """Plain-SGD packs apply W <- W - lr dW where dW is produced; the separate update launch (kept as a
    measuring aid behind an environment variable) must give the same bits, for unsplit weight
    gradients (MLP), split ones (CNN: the update then happens in the reduction kernel), fp32 and bf16."""
    cases = [wl.config2(B=48, D=200, hidden=(72, 40), K=3, steps=3),
             wl.config3(K=2, B=8, size=16, widths=(16, 32, 32), steps=2),
             wl.config5(K=2, B=4, size=16, widths=(16, 32, 32, 64), n_classes=100, steps=2)]
    for w in cases:
        fused = pu.run_gpu(w, keep_first_grads=False)
        fused_keep = pu.run_gpu(w)                       # same kernels, gradients stored as well
        monkeypatch.setenv("PACK_NO_FUSED_UPDATE", "1")
        separate = pu.run_gpu(w)
        monkeypatch.delenv("PACK_NO_FUSED_UPDATE")
        assert separate["launches"] == fused["launches"] + 1
        for k in range(w.K):
            assert np.array_equal(fused["blobs"][k], separate["blobs"][k]), (w.name, k)
            assert np.array_equal(fused_keep["blobs"][k], separate["blobs"][k]), (w.name, k)
            assert np.array_equal(fused_keep["grads"][k], separate["grads"][k]), (w.name, k)
        assert np.array_equal(fused["loss"], separate["loss"])


def test_gradients_of_a_plain_sgd_pack_are_only_kept_on_request():
    from paper_2002_02885_amd import binding
    w = wl.config2(B=16, D=64, hidden=(32,), K=2, steps=1)
    x_dev, y_dev = pu.device_inputs(w)
    pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
    try:
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
        with pytest.raises(binding.PackError) as e:
            pk.read_grads(0)
        assert e.value.status == binding.PACK_EINVAL
        pk.keep_grads(True)
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
        assert np.any(pk.read_grads(0) != 0)
        pk.set_optimizer(1, {"kind": "adam"})            # a member with state: the separate update stores them anyway
        pk.keep_grads(False)
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), w.lr)
        assert np.any(pk.read_grads(0) != 0)
    finally:
        pk.destroy()


def test_the_separate_head_kernels_match_the_oracle_too(monkeypatch):
    """Members with few classes take the one-kernel classifier head; the three separate kernels it
    replaces (last linear forward, loss, its input gradient) stay in use for many classes and behind an
    environment variable, and must pass the same parity check on the same workloads."""
    monkeypatch.setenv("PACK_NO_FUSED_HEAD", "1")
    _check_bf16(wl.config2(B=64, D=256, hidden=(128, 64), K=3, steps=4))
    _check_f32(wl.config3(K=2, B=8, size=16, widths=(16, 32, 32), steps=2))


def test_the_largest_pack_256_members_with_their_own_learning_rates_and_optimisers():
    """PACK_MAX_MODELS members (the per-step tables hold exactly that many entries): a sample of
    members against the oracle, fp32, with every fourth member on Adam (so the separate update runs)
    and, in a second pack, all on plain SGD (so the update in the weight-gradient kernel runs)."""
    K = 256
    rng = np.random.default_rng(123)
    models = [wl.mlp([int(rng.integers(8, 40))], 10) for _ in range(K)]
    batch = [int(b) for b in rng.integers(1, 17, size=K)]
    w = wl.custom("k256", 9, wl.F32, 16, (1, 1, 48), models, batch=batch, steps=2)
    for with_adam in (False, True):
        if with_adam:
            w.meta["optimizers"] = [{"kind": "adam"} if k % 4 == 0 else {"kind": "sgd"} for k in range(K)]
        gpu = pu.run_gpu(w)
        sample = [0, 1, 4, 100, 129, 254, 255]
        for k in sample:
            net = po.Model(models[k], w.in_shape, w.weights[k].astype(np.float64), "exact",
                           opt=(w.meta["optimizers"][k] if with_adam else None))
            for t in range(w.steps):
                l, _, _ = net.sgd_step(w.x[:batch[k]].astype(np.float64), w.labels[:batch[k]], float(w.lr[k]))
                assert abs(gpu["loss"][t, k] - l) <= F32_TOL * abs(l), (with_adam, k, t)
            ref = net.blob()
            scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))
            assert np.max(np.abs(gpu["blobs"][k] - ref) / scale) <= F32_TOL, (with_adam, k)
        assert np.all(np.isfinite(gpu["loss"]))


def test_shortcut_gradient_in_the_first_convolutions_epilogue_equals_the_separate_kernel(monkeypatch):
    """The gradient through a residual shortcut is added by the input-gradient product of the block's
    first convolution (identity: same pixel; subsampling: even pixels of the stride-2 classes or of the
    scalar kernel's rows).  The separate shortcut kernel, kept behind an environment variable, must give
    the same bits: the shortcut's share is exact in the pack dtype and joins the same fp32 sum."""
    cases = [wl.config5(K=2, B=4, size=16, widths=(64, 64, 128), n_classes=10, steps=2),             # aligned: class problems
             wl.config5(K=2, B=3, size=12, widths=(16, 24, 40), n_classes=10, steps=2),              # scalar kernels
             wl.config5(K=2, B=4, size=16, widths=(32, 64), n_classes=10, steps=2, dtype=wl.F32)]
    for w in cases:
        fused = pu.run_gpu(w)
        monkeypatch.setenv("PACK_NO_FUSED_SHORTCUT", "1")
        separate = pu.run_gpu(w)
        monkeypatch.delenv("PACK_NO_FUSED_SHORTCUT")
        assert separate["launches"] > fused["launches"]
        for k in range(w.K):
            assert np.array_equal(fused["grads"][k], separate["grads"][k]), (w.name, w.dtype, k)
            assert np.array_equal(fused["blobs"][k], separate["blobs"][k]), (w.name, w.dtype, k)
