"""GPU parity of packs whose members train on DIFFERENT data (the "Training Data: Different" rows of
the paper's ablation study, Table 2): every slot has its own batch and labels.  Packing is lossless
whatever the members read (Section 2.2), so the oracle is again each member trained alone, now on
its own block; the device-side check is bit-identity with the member trained in a pack of its own
that is fed the same block as a shared batch."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pack_oracle as po
from paper_2002_02885_amd import binding
from tests import parity_util as pu
from tests.test_gpu_dynamic import _check_member, _dataset, _loss_close, _to_dev, _train_static, _weights

pytestmark = pytest.mark.gpu


def _blocks(seed, K, B, T, in_shape, dtype):
    """T steps of K independent batches: X [T, K, B, ...], Y [T, K, B]."""
    X, Y = _dataset(seed, T * K * B, in_shape, dtype)
    return X.reshape((T, K, B) + tuple(in_shape)), Y.reshape(T, K, B)


def test_members_on_different_data_mlp_fp32_against_the_oracle():
    in_shape, B, T = (1, 1, 88), 16, 4
    layers = [wl.mlp([40, 24], 10), [("linear", 33), ("tanh",), ("linear", 10)], wl.mlp([72], 10)]
    batch, lr = [16, 9, 12], np.array([0.05, 0.02, 0.01], dtype=np.float32)
    opts = [{"kind": "sgd"}, {"kind": "momentum", "mu": 0.9}, {"kind": "adam"}]
    X, Y = _blocks(61, 3, B, T, in_shape, wl.F32)
    w0 = [_weights(400 + k, layers[k], in_shape, wl.F32) for k in range(3)]
    nets = [po.Model(layers[k], in_shape, w0[k].astype(np.float64), "exact", opt=opts[k]) for k in range(3)]
    ref_loss = np.zeros((T, 3))
    for t in range(T):
        for k in range(3):
            ref_loss[t, k] = nets[k].sgd_step(X[t, k, :batch[k]].astype(np.float64), Y[t, k, :batch[k]], float(lr[k]))[0]
    pk = binding.Pack(B, in_shape, wl.F32, layers, batch)
    try:
        for k in range(3):
            pk.write_weights(k, w0[k])
            pk.set_optimizer(k, opts[k])
        pk.set_input_mode(True)
        for t in range(T):
            x_dev, y_dev = _to_dev(X[t], wl.F32), torch.from_numpy(np.ascontiguousarray(Y[t])).cuda()
            pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
            loss = pk.read_loss()
            for k in range(3):
                _loss_close(f"step {t} member {k}", loss[k], ref_loss[t, k])
        got = [pk.read_weights(k) for k in range(3)]
    finally:
        pk.destroy()
    for k in range(3):
        print(f"member {k}: displacement error "
              f"{_check_member(f'member {k}', layers[k], in_shape, w0[k], got[k], nets[k].blob(), T):.2e}")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_a_member_on_its_own_block_equals_the_member_alone_on_that_block(dtype):
    """CNNs (each member now has its own im2col copy) and an MLP, with a vacant slot in the middle;
    fp32 is also compared with the oracle."""
    in_shape, B, T = (8, 8, 3), 12, 3
    cnn_a = wl.small_cnn((16, 32, 32), 10)
    cnn_b = [("conv3x3", 16, 2), ("relu",), ("res_begin",), ("conv3x3", 16, 1), ("relu",), ("conv3x3", 16, 1), ("res_end",),
             ("gap",), ("linear", 10)]
    mlp = [("linear", 48), ("leaky_relu",), ("linear", 10)]
    layers, batch, lrs = [cnn_a, mlp, cnn_b, mlp], [12, 7, 10, 12], [0.02, 0.05, 0.03, 0.01]
    X, Y = _blocks(71, 4, B, T, in_shape, dtype)
    w0 = [_weights(500 + k, layers[k], in_shape, dtype) for k in range(4)]
    x_dev = [_to_dev(X[t], dtype) for t in range(T)]
    y_dev = [torch.from_numpy(np.ascontiguousarray(Y[t])).cuda() for t in range(T)]
    pk = binding.Pack(B, in_shape, dtype, layers, batch)
    try:
        for k in range(4):
            pk.write_weights(k, w0[k])
        pk.free(1)                                   # block 1 of every step is then ignored
        pk.set_input_mode(True)
        lr = np.array(lrs, dtype=np.float32)
        for t in range(T):
            pk.step(x_dev[t].data_ptr(), y_dev[t].data_ptr(), lr)
        got = {k: pk.read_weights(k) for k in (0, 2, 3)}
        loss = pk.read_loss()
    finally:
        pk.destroy()
    for k in (0, 2, 3):
        xs = [x_dev[t][k].contiguous() for t in range(T)]
        ys = [y_dev[t][k].contiguous() for t in range(T)]
        want, _ = _train_static(dtype, in_shape, B, layers[k], batch[k], w0[k], {"kind": "sgd"}, lrs[k], xs, ys, range(T))
        assert np.array_equal(got[k], want), f"member {k}"
        if dtype == wl.F32:
            net = po.Model(layers[k], in_shape, w0[k].astype(np.float64), "exact")
            for t in range(T):
                l = net.sgd_step(X[t, k, :batch[k]].astype(np.float64), Y[t, k, :batch[k]], lrs[k])[0]
            _loss_close(f"member {k} last loss", loss[k], l)
            _check_member(f"member {k}", layers[k], in_shape, w0[k], got[k], net.blob(), T)


def test_switching_the_input_mode_keeps_the_members_state():
    """Shared for two steps, per-member for two steps with every block equal to the shared batch,
    shared again: the same bits as four... five shared steps."""
    in_shape, B = (1, 1, 64), 8
    layers = [wl.mlp([32], 10), wl.mlp([16, 16], 10)]
    X, Y = _dataset(81, B, in_shape, wl.BF16)
    x1, y1 = _to_dev(X, wl.BF16), torch.from_numpy(Y).cuda()
    x2, y2 = torch.stack([x1, x1]).contiguous(), torch.stack([y1, y1]).contiguous()
    w0 = [_weights(600 + k, layers[k], in_shape, wl.BF16) for k in range(2)]
    lr = np.array([0.05, 0.02], dtype=np.float32)
    opt = {"kind": "momentum", "mu": 0.5}

    def run(switch):
        pk = binding.Pack(B, in_shape, wl.BF16, layers, [8, 5])
        try:
            for k in range(2):
                pk.write_weights(k, w0[k])
                pk.set_optimizer(k, opt)
            for t in range(5):
                per_member = switch and t in (2, 3)
                pk.set_input_mode(per_member)
                if per_member:
                    pk.step(x2.data_ptr(), y2.data_ptr(), lr)
                else:
                    pk.step(x1.data_ptr(), y1.data_ptr(), lr)
            return [pk.read_weights(k) for k in range(2)], [pk.read_opt_state(k, 0)[0] for k in range(2)]
        finally:
            pk.destroy()

    a, b = run(False), run(True)
    for k in range(2):
        assert np.array_equal(a[0][k], b[0][k]) and np.array_equal(a[1][k], b[1][k])
    pk = binding.Pack(B, in_shape, wl.BF16, layers, [8, 5])
    try:
        with pytest.raises(binding.PackError) as e:
            binding._check(binding.lib().pack_set_input_mode(pk._h, 2))
        assert e.value.status == binding.PACK_EINVAL
    finally:
        pk.destroy()
