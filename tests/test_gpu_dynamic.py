"""GPU parity of a pack that changes while it trains: members leave and join (paper Section 3.3,
`load` / `free` on a live pack), the shared batch is re-sliced, and a whole epoch over members
with different batch sizes follows the progress-tracking schedule of Section 3.2.

The oracle needs no new arithmetic for any of this: packing is lossless (Section 2.2), so whatever
happens to the rest of the pack, a member's weights are those of the member trained alone on the
rows it was given.  The tests therefore train every member separately in float64 on exactly those
rows and compare (1e-4 relative for fp32 packs), and also check the stronger device-side property
that a member's bits do not depend on the pack's history."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pack_oracle as po
from oracle import schedule_oracle as so
from paper_2002_02885_amd import binding
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

TOL = pu.TOL[wl.F32]


def _dataset(seed, n, in_shape, dtype, n_classes=10):
    """n seeded samples (the stand-in for the paper's datasets) + one spare workload for weights."""
    w = wl.custom("dataset", seed, dtype, n, in_shape, [wl.mlp([8], n_classes)], n_classes=n_classes)
    return w.x, w.labels


def _to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == wl.BF16:
        t = t.to(torch.bfloat16)
    return t.cuda().contiguous()


def _weights(seed, layers, in_shape, dtype):
    return wl.draw_weights(np.random.default_rng(np.random.PCG64(seed)), layers, in_shape, dtype)


def _check_member(name, layers, in_shape, w0, gpu_blob, ref_blob, steps, tol=TOL):
    """Displacement W_T - W_0 per tensor, infinity norm relative to the reference displacement."""
    gw, rw, w0 = np.asarray(gpu_blob, np.float64), np.asarray(ref_blob, np.float64), np.asarray(w0, np.float64)
    worst = 0.0
    for tname, s in pu.tensor_slices(layers, in_shape):
        dg, dr = gw[s] - w0[s], rw[s] - w0[s]
        floor = 2.0 ** -23 * steps * np.max(np.abs(w0[s])) / max(np.max(np.abs(dr)), 1e-300)
        e = pu.rel_inf(dg, dr)
        assert e <= tol + floor, f"{name} {tname}: displacement error {e} > {tol + floor}"
        worst = max(worst, e)
    return worst


def _loss_close(name, got, want, tol=TOL):
    assert abs(got - want) <= tol * abs(want), f"{name}: loss {got} vs {want}"


MLP_A = wl.mlp([40, 33], 10)
MLP_B = [("linear", 64), ("tanh",), ("linear", 10)]
MLP_C = wl.mlp([17, 29, 20], 10)
MLP_D = [("linear", 48), ("leaky_relu",), ("linear", 24), ("relu",), ("linear", 10)]
OPT_A = {"kind": "adam", "beta1": 0.9, "beta2": 0.99, "eps": 1e-6}
OPT_C = {"kind": "momentum", "mu": 0.8}
OPT_D = {"kind": "adagrad", "acc0": 0.1}


def test_members_leave_and_join_a_live_pack_fp32():
    in_shape, B, T = (1, 1, 96), 24, 8
    X, Y = _dataset(11, B * T, in_shape, wl.F32)
    xb = [X[t * B:(t + 1) * B] for t in range(T)]
    yb = [Y[t * B:(t + 1) * B] for t in range(T)]
    x_dev = [_to_dev(x, wl.F32) for x in xb]
    y_dev = [torch.from_numpy(y).cuda() for y in yb]
    layers = {"A": MLP_A, "B": MLP_B, "C": MLP_C, "D": MLP_D}
    batch = {"A": 24, "B": 16, "C": 9, "D": 20}
    lr = {"A": 0.01, "B": 0.05, "C": 0.02, "D": 0.03}
    opts = {"A": OPT_A, "B": {"kind": "sgd"}, "C": OPT_C, "D": OPT_D}
    w0 = {n: _weights(100 + i, layers[n], in_shape, wl.F32) for i, n in enumerate("ABCD")}
    alive = {"A": range(0, 8), "B": range(0, 3), "C": range(0, 8), "D": range(5, 8)}

    # oracle: every member alone, on the rows it was given, for the steps it was in the pack
    ref_loss, ref_blob = {}, {}
    for n in "ABCD":
        net = po.Model(layers[n], in_shape, w0[n].astype(np.float64), "exact", opt=opts[n])
        ref_loss[n] = {}
        for t in alive[n]:
            l, _, _ = net.sgd_step(xb[t][:batch[n]].astype(np.float64), yb[t][:batch[n]], lr[n])
            ref_loss[n][t] = l
        ref_blob[n] = net.blob()

    pk = binding.Pack(B, in_shape, wl.F32, [layers["A"], layers["B"], layers["C"]], [batch["A"], batch["B"], batch["C"]])
    try:
        slot = {"A": 0, "B": 1, "C": 2}
        for n, k in slot.items():
            pk.write_weights(k, w0[n])
            pk.set_optimizer(k, opts[n])
        got_blob = {}

        def run(t):
            lrs = np.zeros(pk.K, dtype=np.float32)
            for n, k in slot.items():
                lrs[k] = lr[n]
            pk.step(x_dev[t].data_ptr(), y_dev[t].data_ptr(), lrs)
            loss = pk.read_loss()
            for n, k in slot.items():
                _loss_close(f"step {t} member {n}", loss[k], ref_loss[n][t])
            for k in range(pk.K):
                if k not in slot.values():
                    assert loss[k] == 0.0

        for t in range(0, 3):
            run(t)
        got_blob["B"] = pk.read_weights(slot["B"])          # free's checkpoint
        bytes_before = pk.device_bytes()
        pk.free(slot.pop("B"))
        assert pk.K == 3 and pk.batch == [24, 0, 9] and pk.device_bytes() < bytes_before
        with pytest.raises(binding.PackError):
            pk.read_weights(1)
        for t in range(3, 5):
            run(t)
        k_new = pk.load(layers["D"], batch["D"], seed=5)
        assert k_new == 1 and pk.batch == [24, 20, 9]
        slot["D"] = k_new
        pk.write_weights(k_new, w0["D"])
        pk.set_optimizer(k_new, opts["D"])
        for t in range(5, 8):
            run(t)
        for n, k in slot.items():
            got_blob[n] = pk.read_weights(k)
        _, adam_steps = pk.read_opt_state(slot["A"], 0)
        assert adam_steps == 8                               # the step counter travelled with the member
    finally:
        pk.destroy()
    for n in "ABCD":
        worst = _check_member(n, layers[n], in_shape, w0[n], got_blob[n], ref_blob[n], len(alive[n]))
        print(f"member {n}: displacement error {worst:.2e}")


def _train_static(dtype, in_shape, B, layers, batch, w0, opt, lr, x_dev, y_dev, steps):
    pk = binding.Pack(B, in_shape, dtype, [layers], [batch])
    try:
        pk.write_weights(0, w0)
        pk.set_optimizer(0, opt)
        for t in steps:
            pk.step(x_dev[t].data_ptr(), y_dev[t].data_ptr(), np.array([lr], dtype=np.float32))
        state = pk.read_opt_state(0, 0)[0] if opt["kind"] != "sgd" else None
        return pk.read_weights(0), state
    finally:
        pk.destroy()


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_a_members_bits_do_not_depend_on_the_packs_history(dtype):
    """A small CNN (shared im2col input, transposed-weight copy, split weight-gradient reduction) and
    an MLP stay in a pack while a third member leaves, another joins and the batch is re-sliced;
    both end with exactly the bits they reach when trained alone in a pack that never changes."""
    in_shape, B, T = (8, 8, 3), 16, 6
    X, Y = _dataset(21, B * T, in_shape, dtype)
    x_dev = [_to_dev(X[t * B:(t + 1) * B], dtype) for t in range(T)]
    y_dev = [torch.from_numpy(Y[t * B:(t + 1) * B]).cuda() for t in range(T)]
    cnn = [("conv3x3", 16, 1), ("relu",), ("res_begin",), ("conv3x3", 16, 1), ("relu",), ("conv3x3", 16, 1), ("res_end",),
           ("conv3x3", 32, 2), ("relu",), ("gap",), ("linear", 10)]
    mlp = [("linear", 40), ("sigmoid",), ("linear", 10)]
    other = wl.small_cnn((16, 32, 32), 10)
    w_cnn, w_mlp = _weights(1, cnn, in_shape, dtype), _weights(2, mlp, in_shape, dtype)
    want_cnn, want_cnn_state = _train_static(dtype, in_shape, B, cnn, 12, w_cnn, OPT_C, 0.02, x_dev, y_dev, range(T))
    want_mlp, _ = _train_static(dtype, in_shape, B, mlp, 16, w_mlp, {"kind": "sgd"}, 0.05, x_dev, y_dev, range(T))

    pk = binding.Pack(B, in_shape, dtype, [other, cnn, mlp], [16, 12, 16])
    try:
        pk.write_weights(1, w_cnn)
        pk.write_weights(2, w_mlp)
        pk.set_optimizer(1, OPT_C)
        lr3 = np.array([0.01, 0.02, 0.05], dtype=np.float32)
        for t in range(0, 2):
            pk.step(x_dev[t].data_ptr(), y_dev[t].data_ptr(), lr3)
        pk.free(0)
        pk.step(x_dev[2].data_ptr(), y_dev[2].data_ptr(), lr3)
        k = pk.load(wl.mlp([24], 10), 5, seed=3)
        assert k == 0
        k = pk.load(other, 16, seed=4)
        assert k == 3 and pk.K == 4
        lr4 = np.array([0.1, 0.02, 0.05, 0.01], dtype=np.float32)
        pk.step(x_dev[3].data_ptr(), y_dev[3].data_ptr(), lr4)
        pk.set_batch(16, [3, 12, 16, 8])                     # others re-sliced, the two watched members unchanged
        pk.step(x_dev[4].data_ptr(), y_dev[4].data_ptr(), lr4)
        pk.free(3)
        pk.step(x_dev[5].data_ptr(), y_dev[5].data_ptr(), lr4)
        assert np.array_equal(pk.read_weights(1), want_cnn)
        assert np.array_equal(pk.read_opt_state(1, 0)[0], want_cnn_state)
        assert np.array_equal(pk.read_weights(2), want_mlp)
    finally:
        pk.destroy()


def test_epoch_with_different_batch_sizes_follows_the_progress_schedule_fp32():
    """One epoch over 50 samples with batch sizes 10, 4 and 7 (phases end in short batches): the
    device path takes its steps from the library's schedule, assembles each shared batch with the
    gather kernel, frees members as they finish and re-slices the batch; the oracle trains each
    member alone along the oracle's own schedule."""
    in_shape, N = (1, 1, 72), 50
    batch = [10, 4, 7]
    layers = [wl.mlp([32, 16], 10), [("linear", 24), ("tanh",), ("linear", 10)], wl.mlp([20], 10)]
    opts = [{"kind": "sgd"}, OPT_A, OPT_C]
    lr = np.array([0.05, 0.01, 0.03], dtype=np.float32)
    X, Y = _dataset(31, N, in_shape, wl.F32)
    w0 = [_weights(300 + k, layers[k], in_shape, wl.F32) for k in range(3)]

    steps = so.epoch_schedule(N, batch)
    nets = [po.Model(layers[k], in_shape, w0[k].astype(np.float64), "exact", opt=opts[k]) for k in range(3)]
    n_steps = [0, 0, 0]
    for st in steps:
        for k in range(3):
            r = st["rows"][k]
            if r:
                idx = st["idx"][:r]
                nets[k].sgd_step(X[idx].astype(np.float64), Y[idx], float(lr[k]))
                n_steps[k] += 1

    data_dev, labels_dev = _to_dev(X, wl.F32), torch.from_numpy(Y).cuda()
    x_buf = torch.zeros((max(batch),) + in_shape, dtype=torch.float32, device="cuda")
    y_buf = torch.zeros(max(batch), dtype=torch.int32, device="cuda")
    pk = binding.Pack(max(batch), in_shape, wl.F32, layers, batch)
    sched = binding.Schedule(N, batch)
    got, taken = {}, 0
    try:
        for k in range(3):
            pk.write_weights(k, w0[k])
            pk.set_optimizer(k, opts[k])
        while True:
            nxt = sched.next()
            if nxt is None:
                break
            idx, rows_k, lead = nxt
            assert list(idx) == steps[taken]["idx"] and list(rows_k) == steps[taken]["rows"] and lead == steps[taken]["lead"]
            for k in range(3):
                if rows_k[k] == 0 and pk.batch[k] != 0:      # finished: checkpoint, then free
                    got[k] = pk.read_weights(k)
                    pk.free(k)
            pk.set_batch(len(idx), [int(r) for r in rows_k])
            idx_dev = torch.from_numpy(idx).cuda()
            pk.gather_batch(data_dev.data_ptr(), labels_dev.data_ptr(), N, idx_dev.data_ptr(), len(idx),
                            x_buf.data_ptr(), y_buf.data_ptr())
            pk.step(x_buf.data_ptr(), y_buf.data_ptr(), lr)
            pk.read_loss()
            taken += 1
        for k in range(3):
            if pk.batch[k] != 0:
                got[k] = pk.read_weights(k)
        assert list(sched.used()) == [N, N, N] and taken == len(steps)
    finally:
        sched.destroy()
        pk.destroy()
    for k in range(3):
        worst = _check_member(f"member {k}", layers[k], in_shape, w0[k], got[k], nets[k].blob(), n_steps[k])
        print(f"member {k}: {n_steps[k]} steps, displacement error {worst:.2e}")


@pytest.mark.parametrize("dtype,in_shape", [(wl.F32, (4, 4, 3)), (wl.BF16, (4, 4, 3)), (wl.F32, (1, 1, 7)), (wl.BF16, (1, 1, 7)),
                                            (wl.BF16, (32, 32, 3))])
def test_gather_batch_is_a_bit_exact_row_gather(dtype, in_shape):
    """Against numpy's fancy indexing, for row sizes that take the 16-, 4- and 2-byte paths."""
    N, B = 300, 64
    X, Y = _dataset(41, N, in_shape, dtype)
    rng = np.random.default_rng(5)
    data_dev, labels_dev = _to_dev(X, dtype), torch.from_numpy(Y).cuda()
    tdtype = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    pk = binding.Pack(B, in_shape, dtype, [wl.mlp([8], 10)], [B])
    try:
        for rows in (B, 37, 1, 0):
            idx = rng.integers(0, N, size=rows).astype(np.int64)
            x_buf = torch.full((B,) + in_shape, 7.0, dtype=tdtype, device="cuda")
            y_buf = torch.full((B,), -5, dtype=torch.int32, device="cuda")
            idx_dev = torch.from_numpy(idx).cuda() if rows else torch.zeros(1, dtype=torch.int64, device="cuda")
            pk.gather_batch(data_dev.data_ptr(), labels_dev.data_ptr(), N, idx_dev.data_ptr(), rows, x_buf.data_ptr(), y_buf.data_ptr())
            torch.cuda.synchronize()
            got_x, got_y = x_buf.float().cpu().numpy(), y_buf.cpu().numpy()
            assert np.array_equal(got_x[:rows], X[idx]) and np.array_equal(got_y[:rows], Y[idx])
            assert np.all(got_x[rows:] == 7.0) and np.all(got_y[rows:] == -5)     # rows beyond `rows` untouched
        # an index outside the dataset: zeros, label -1, reported at the next read of the losses
        idx = np.array([3, N, 5, -1], dtype=np.int64)
        x_buf = torch.full((B,) + in_shape, 7.0, dtype=tdtype, device="cuda")
        y_buf = torch.full((B,), -5, dtype=torch.int32, device="cuda")
        idx_dev = torch.from_numpy(idx).cuda()
        pk.gather_batch(data_dev.data_ptr(), labels_dev.data_ptr(), N, idx_dev.data_ptr(), 4, x_buf.data_ptr(), y_buf.data_ptr())
        torch.cuda.synchronize()
        got_x, got_y = x_buf.float().cpu().numpy(), y_buf.cpu().numpy()
        assert np.array_equal(got_x[0], X[3]) and np.array_equal(got_x[2], X[5])
        assert np.all(got_x[1] == 0) and np.all(got_x[3] == 0) and list(got_y[:4]) == [Y[3], -1, Y[5], -1]
        pk.read_loss(allow_label_error=True)
        assert pk.last_status == binding.PACK_EINDEX
        pk.read_loss()                                           # the flag is cleared by the read
    finally:
        pk.destroy()


def test_dynamic_calls_reject_bad_arguments_and_leave_the_pack_unchanged():
    in_shape, B = (1, 1, 40), 12
    X, Y = _dataset(51, B, in_shape, wl.F32)
    x_dev, y_dev = _to_dev(X, wl.F32), torch.from_numpy(Y).cuda()
    w0 = _weights(7, MLP_A, in_shape, wl.F32)
    lr = np.array([0.05], dtype=np.float32)
    want, _ = _train_static(wl.F32, in_shape, B, MLP_A, 12, w0, {"kind": "sgd"}, 0.05, [x_dev], [y_dev], [0, 0])
    pk = binding.Pack(B, in_shape, wl.F32, [MLP_A], [12])
    try:
        pk.write_weights(0, w0)
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
        for bad in (lambda: pk.free(1), lambda: pk.free(-1), lambda: pk.load(MLP_B, B + 1), lambda: pk.load(MLP_B, 0),
                    lambda: pk.load([("relu",), ("linear", 10)], 4), lambda: pk.set_batch(8, [9]),
                    lambda: pk.set_batch(0, [1]),
                    lambda: pk.gather_batch(x_dev.data_ptr(), y_dev.data_ptr(), B, y_dev.data_ptr(), B + 1, x_dev.data_ptr(), y_dev.data_ptr())):
            with pytest.raises(binding.PackError) as e:
                bad()
            assert e.value.status in (binding.PACK_EINVAL, binding.PACK_ESHAPE)
        assert pk.K == 1 and pk.batch == [12]
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
        assert np.array_equal(pk.read_weights(0), want)
        # the last member may leave too: the pack is empty, a step does nothing, and it can be filled again
        pk.free(0)
        assert pk.num_launches() == 0
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
        assert list(pk.read_loss()) == [0.0]
        assert pk.load(MLP_A, 12) == 0
        pk.write_weights(0, w0)
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
        pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
        assert np.array_equal(pk.read_weights(0), want)
    finally:
        pk.destroy()
