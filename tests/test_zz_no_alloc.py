"""The step that allocates nothing (pack_step_static), called through the C ABI, against pack_step: the same
kernels with the partial sums of split weight gradients in the library's static scratch array instead of the
pack's own workspace, so the results must agree bit for bit.  Two calls in a row share the array, the second
from a smaller pack."""
import numpy as np
import pytest

import workloads as wl
from paper_2002_02885_amd import binding
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _twins(w):
    out = []
    for _ in range(2):
        pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
        for k in range(w.K):
            pk.write_weights(k, w.weights[k])
        out.append(pk)
    return out


def _state(pk, w):
    return [pk.read_weights(k).view(np.uint32) for k in range(w.K)], pk.read_loss(), [pk.read_pred(k) for k in range(w.K)]


def test_static_scratch_step_equals_the_allocating_step_on_two_calls_in_a_row():
    big = wl.config3(K=3, B=16, size=32, widths=(32, 64, 128), steps=2)                        # fp32, split convolution gradients
    small = wl.config5(K=2, B=4, size=16, widths=(64, 64), n_classes=10, steps=2)              # bf16, a smaller pack
    assert binding.static_scratch_bytes() == 128 << 20
    packs = []
    try:
        for w in (big, small):
            ref, sta = _twins(w)
            packs += [ref, sta]
            assert 0 < ref.workspace_bytes() == sta.workspace_bytes() <= binding.static_scratch_bytes()
            x, y = pu.device_inputs(w)
            for _ in range(w.steps):
                ref.step(x.data_ptr(), y.data_ptr(), w.lr)
                sta.step_static(x.data_ptr(), y.data_ptr(), w.lr)
            (wr, lr_, pr), (ws, ls, ps) = _state(ref, w), _state(sta, w)
            for a, b in zip(wr, ws):
                assert np.array_equal(a, b), w.name
            assert np.array_equal(lr_, ls) and all(np.array_equal(a, b) for a, b in zip(pr, ps))
            assert np.all(np.isfinite(ls))
        # the two kinds of step may alternate on one pack (one stream: no overlap)
        ref, sta = packs[0], packs[1]
        x, y = pu.device_inputs(big)
        ref.step(x.data_ptr(), y.data_ptr(), big.lr)
        ref.step_static(x.data_ptr(), y.data_ptr(), big.lr)
        sta.step_static(x.data_ptr(), y.data_ptr(), big.lr)
        sta.step(x.data_ptr(), y.data_ptr(), big.lr)
        for a, b in zip(_state(ref, big)[0], _state(sta, big)[0]):
            assert np.array_equal(a, b)
    finally:
        for pk in packs:
            pk.destroy()


def test_static_scratch_step_rejects_what_does_not_fit_and_a_pack_that_is_being_timed():
    w = wl.config5(K=1, B=2, size=16, widths=(64, 64), n_classes=10, steps=1)
    x, y = pu.device_inputs(w)
    pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
    try:
        pk.profile_start(-1)
        with pytest.raises(binding.PackError) as e:
            pk.step_static(x.data_ptr(), y.data_ptr(), w.lr)
        assert e.value.status == binding.PACK_EINVAL
        pk.profile_stop()
        pk.step_static(x.data_ptr(), y.data_ptr(), w.lr)
        assert np.all(np.isfinite(pk.read_loss()))
    finally:
        pk.destroy()
    # six members of the largest configuration need more scratch than the array holds: rejected, nothing launched
    full = wl.config5()
    models, batch = [full.models[0]] * 6, [full.batch[0]] * 6
    pk = binding.Pack(full.B, full.in_shape, full.dtype, models, batch)
    try:
        assert pk.workspace_bytes() > binding.static_scratch_bytes()
        xf, yf = pu.device_inputs(full)
        with pytest.raises(binding.PackError) as e:
            pk.step_static(xf.data_ptr(), yf.data_ptr(), np.full(6, 1e-3, dtype=np.float32))
        assert e.value.status == binding.PACK_ENOMEM and "static" in str(e.value)
    finally:
        pk.destroy()
