"""Shared helpers of the GPU parity tests: run a workload through the C ABI, run the same
workload through the CPU oracle, and compare per member and per tensor."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from oracle import pack_oracle as po
from paper_2002_02885_amd import binding

TOL = {wl.F32: 1e-4, wl.BF16: 2e-2}    # max relative error the two paths may differ by


def device_inputs(w: wl.PackWorkload):
    """The shared batch and labels as device tensors of the pack's element type."""
    x = torch.from_numpy(w.x)
    if w.dtype == wl.BF16:
        x = x.to(torch.bfloat16)           # exact: the values are bf16-representable
    return x.cuda().contiguous(), torch.from_numpy(w.labels).cuda().contiguous()


def run_gpu(w: wl.PackWorkload, steps=None, lr=None, x_dev=None, y_dev=None, keep_first_grads=True):
    """Trains `w` for `steps` steps through libpack; returns dict(loss [steps,K], grads (step 1),
    logits (step 1), pred (last step), blobs (after the last step), launches)."""
    steps = w.steps if steps is None else steps
    lr = w.lr if lr is None else np.asarray(lr, dtype=np.float32)
    pk = binding.Pack(w.B, w.in_shape, w.dtype, w.models, w.batch)
    try:
        for k in range(w.K):
            pk.write_weights(k, w.weights[k])
        if x_dev is None:
            x_dev, y_dev = device_inputs(w)
        loss = np.zeros((steps, w.K), dtype=np.float64)
        grads = logits = pred_first = None
        for t in range(steps):
            pk.step(x_dev.data_ptr(), y_dev.data_ptr(), lr)
            loss[t] = pk.read_loss()
            if t == 0 and keep_first_grads:
                grads = [pk.read_grads(k) for k in range(w.K)]
                logits = [pk.read_logits(k) for k in range(w.K)]
                pred_first = [pk.read_pred(k) for k in range(w.K)]
        out = {"loss": loss, "grads": grads, "logits": logits, "pred_first": pred_first,
               "pred": [pk.read_pred(k) for k in range(w.K)],
               "blobs": [pk.read_weights(k) for k in range(w.K)],
               "launches": pk.num_launches(), "device_bytes": pk.device_bytes()}
    finally:
        pk.destroy()
    return out


def run_oracle(w: wl.PackWorkload, steps=None, mode="exact", lr=None):
    steps = w.steps if steps is None else steps
    lr = w.lr if lr is None else lr
    return po.train_pack(w.models, w.in_shape, [b.astype(np.float64) for b in w.weights], w.batch,
                         np.asarray(lr, dtype=np.float64), w.x.astype(np.float64), w.labels, steps,
                         mode=mode, keep_grads=True)


def tensor_slices(layers, in_shape):
    out, off = [], 0
    for kind, ws, bs, _ in wl.param_shapes(layers, in_shape):
        nw, nb = int(np.prod(ws)), int(np.prod(bs))
        out.append((f"{kind}{len(out) // 2}.W", slice(off, off + nw)))
        out.append((f"{kind}{len(out) // 2}.b", slice(off + nw, off + nw + nb)))
        off += nw + nb
    return out


def rel_inf(g, r):
    den = np.max(np.abs(r))
    return float(np.max(np.abs(g - r)) / den) if den > 0 else float(np.max(np.abs(g - r)))


def rel_l2(g, r):
    den = np.linalg.norm(r)
    return float(np.linalg.norm(g - r) / den) if den > 0 else float(np.linalg.norm(g - r))


def compare(w: wl.PackWorkload, gpu: dict, ref: dict, tol: float, what=("loss", "grads", "disp", "weights"),
            label=""):
    """Asserts agreement and returns the worst figures seen.  Gradients and the displacement
    W_T - W_0 are compared per tensor in the infinity norm and the 2-norm (raw weights barely
    move at small learning rates, so agreement of raw weights alone would be vacuous)."""
    worst = {"loss": 0.0, "grads_inf": 0.0, "grads_l2": 0.0, "disp_inf": 0.0, "disp_l2": 0.0, "weights": 0.0}
    steps = gpu["loss"].shape[0]
    for k in range(w.K):
        tag = f"{label}{w.name} member {k}"
        if "loss" in what:
            for t in range(steps):
                e = abs(gpu["loss"][t, k] - ref["loss"][t, k]) / max(abs(ref["loss"][t, k]), 1e-30)
                worst["loss"] = max(worst["loss"], e)
                assert e <= tol, f"{tag}: loss step {t}: gpu {gpu['loss'][t, k]} oracle {ref['loss'][t, k]} rel {e}"
        sl = tensor_slices(w.models[k], w.in_shape)
        if "grads" in what and gpu["grads"] is not None:
            g, r = gpu["grads"][k].astype(np.float64), ref["grads"][0][k]
            assert g.shape == r.shape
            for name, s in sl:
                ei, e2 = rel_inf(g[s], r[s]), rel_l2(g[s], r[s])
                worst["grads_inf"] = max(worst["grads_inf"], ei)
                worst["grads_l2"] = max(worst["grads_l2"], e2)
                assert ei <= tol and e2 <= tol, f"{tag}: grad {name}: inf {ei} l2 {e2}"
        w0 = w.weights[k].astype(np.float64)
        gw, rw = gpu["blobs"][k].astype(np.float64), ref["blobs"][k]
        if "disp" in what and float(w.lr[k]) != 0.0:
            for name, s in sl:
                dg, dr = gw[s] - w0[s], rw[s] - w0[s]
                # the fp32 master rounds each update to 2^-24 of the weight: allow for it
                floor = 2.0 ** -23 * steps * np.max(np.abs(w0[s])) / max(np.max(np.abs(dr)), 1e-300)
                ei, e2 = rel_inf(dg, dr), rel_l2(dg, dr)
                worst["disp_inf"] = max(worst["disp_inf"], ei)
                worst["disp_l2"] = max(worst["disp_l2"], e2)
                assert ei <= tol + floor and e2 <= tol + floor, f"{tag}: displacement {name}: inf {ei} l2 {e2} (floor {floor})"
        if "weights" in what:
            scale = np.maximum(np.abs(rw), np.sqrt(np.mean(rw * rw)))
            e = float(np.max(np.abs(gw - rw) / scale))
            worst["weights"] = max(worst["weights"], e)
            assert e <= tol, f"{tag}: weights: {e}"
    return worst


def compare_pred(w: wl.PackWorkload, gpu_pred, gpu_logits, ref_pred, tol: float):
    """argmax must agree exactly on every row whose top-2 logit gap is resolvable at the
    comparison tolerance; returns (rows compared, rows skipped as unresolvable)."""
    compared = skipped = 0
    for k in range(w.K):
        lg = gpu_logits[k].astype(np.float64)
        srt = np.sort(lg, axis=1)
        gap = srt[:, -1] - srt[:, -2] if lg.shape[1] > 1 else np.full(lg.shape[0], np.inf)
        ok = gap > 4 * tol * np.max(np.abs(lg))
        assert gpu_pred[k].dtype == np.int32
        assert np.array_equal(gpu_pred[k][ok], ref_pred[k][ok]), f"{w.name} member {k}: argmax differs"
        compared += int(ok.sum())
        skipped += int((~ok).sum())
    return compared, skipped
