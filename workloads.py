"""Seeded synthetic inputs for packed training: architectures, initial weights, learning rates,
the shared batch and its labels.

This module only draws random numbers and arranges them into arrays.  It contains none of the
training arithmetic and is imported by the CPU oracle's tests and by the GPU binding's callers
alike, so that both sides see the same data.  The synthetic batches stand in for the image
datasets the paper trains on (Section 4.1 uses ImageNet crops, Section 5.3 uses CIFAR-10): they
keep the tensor shapes (784 / 3072 flat inputs, 32x32x3 and 64x64x3 NHWC images, 10 or 100
classes) but every value is drawn from a seeded numpy PCG64 generator.

Layer lists use plain tuples so that neither consumer needs the other's types:

    ("linear", out_features)        fully connected layer with bias
    ("conv3x3", out_channels, stride)   3x3 convolution, zero padding 1, with bias
    ("relu",)                       max(z, 0)
    ("gap",)                        global average pool over H x W
    ("res_begin",)                  remember the current tensor as the shortcut source
    ("res_end",)                    y = relu(current + shortcut(source))

Flat per-model weight blob (fp32): layers in order; linear = W[out][in] then b[out];
conv = W[Cout][Cin][3][3] then b[Cout].  A linear layer applied to an image flattens it in
NHWC order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

Layer = Tuple
F32 = "f32"
BF16 = "bf16"


@dataclass
class PackWorkload:
    """Everything one packed training run needs, as plain arrays."""
    name: str
    dtype: str                      # F32 or BF16 (bf16 operands, fp32 accumulate and master)
    B: int                          # rows of the shared batch
    in_shape: Tuple[int, int, int]  # (H, W, C); MLP input is (1, 1, D)
    models: List[List[Layer]]       # K layer lists
    batch: List[int]                # b_k <= B: model k trains on rows [0, b_k)
    weights: List[np.ndarray]       # K flat fp32 blobs (bf16-representable when dtype is BF16)
    lr: np.ndarray                  # fp32 [K]
    x: np.ndarray                   # fp32 [B, H, W, C] (bf16-representable when dtype is BF16)
    labels: np.ndarray              # int32 [B]
    steps: int                      # number of steps the parity run takes
    n_classes: int
    meta: dict = field(default_factory=dict)

    @property
    def K(self) -> int:
        return len(self.models)


# ----------------------------------------------------------------------------------------------
# shape bookkeeping (no arithmetic of the method: only sizes)
# ----------------------------------------------------------------------------------------------

def conv_out_size(n: int, stride: int) -> int:
    """Spatial output size of a 3x3 convolution with zero padding 1."""
    return (n + 2 - 3) // stride + 1


def param_shapes(layers: Sequence[Layer], in_shape: Tuple[int, int, int]):
    """List of (kind, W_shape, b_shape, fan_in) for every parameterised layer, in order."""
    h, w, c = in_shape
    out = []
    for op in layers:
        kind = op[0]
        if kind == "linear":
            fan_in = h * w * c
            out.append(("linear", (op[1], fan_in), (op[1],), fan_in))
            h, w, c = 1, 1, op[1]
        elif kind == "conv3x3":
            fan_in = 9 * c
            out.append(("conv3x3", (op[1], c, 3, 3), (op[1],), fan_in))
            h, w, c = conv_out_size(h, op[2]), conv_out_size(w, op[2]), op[1]
        elif kind == "gap":
            h, w = 1, 1
        elif kind in ("relu", "leaky_relu", "sigmoid", "tanh", "res_begin", "res_end"):
            pass
        else:
            raise ValueError(f"unknown layer {op!r}")
    return out


def num_params(layers: Sequence[Layer], in_shape: Tuple[int, int, int]) -> int:
    return sum(int(np.prod(ws)) + int(np.prod(bs)) for _, ws, bs, _ in param_shapes(layers, in_shape))


def split_blob(blob: np.ndarray, layers: Sequence[Layer], in_shape: Tuple[int, int, int]):
    """Views (W, b) into a flat blob, one pair per parameterised layer."""
    pairs, off = [], 0
    for _, ws, bs, _ in param_shapes(layers, in_shape):
        nw, nb = int(np.prod(ws)), int(np.prod(bs))
        pairs.append((blob[off:off + nw].reshape(ws), blob[off + nw:off + nw + nb].reshape(bs)))
        off += nw + nb
    assert off == blob.size
    return pairs


def step_flops(layers: Sequence[Layer], in_shape: Tuple[int, int, int], rows: int) -> int:
    """Multiply-add work of one training step of one model, counted as 2*m*n*k for each of the
    forward product, the weight-gradient product and the input-gradient product; the
    input-gradient product of the first parameterised layer is not needed (its input is data)."""
    h, w, c = in_shape
    total, first = 0, True
    for op in layers:
        if op[0] == "linear":
            f = 2 * rows * (h * w * c) * op[1]
            total += f * (2 if first else 3)
            first = False
            h, w, c = 1, 1, op[1]
        elif op[0] == "conv3x3":
            ho, wo = conv_out_size(h, op[2]), conv_out_size(w, op[2])
            f = 2 * rows * ho * wo * op[1] * 9 * c
            total += f * (2 if first else 3)
            first = False
            h, w, c = ho, wo, op[1]
        elif op[0] == "gap":
            h, w = 1, 1
    return total


# ----------------------------------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------------------------------

def to_bf16_representable(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them as fp32."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable fp32 values (the upper half of each word)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16)


def draw_weights(rng: np.random.Generator, layers, in_shape, dtype) -> np.ndarray:
    """Kaiming-uniform: W ~ U(-sqrt(6/fan_in), +sqrt(6/fan_in)), b ~ U(-1/sqrt(fan_in), +...)."""
    parts = []
    for _, ws, bs, fan_in in param_shapes(layers, in_shape):
        bw = np.sqrt(6.0 / fan_in)
        bb = 1.0 / np.sqrt(fan_in)
        parts.append(rng.uniform(-bw, bw, size=int(np.prod(ws))).astype(np.float32))
        parts.append(rng.uniform(-bb, bb, size=int(np.prod(bs))).astype(np.float32))
    blob = np.concatenate(parts)
    return to_bf16_representable(blob) if dtype == BF16 else blob


def _finish(name, dtype, B, in_shape, models, batch, lr, rng, pixel, n_classes, steps, meta=None):
    weights = [draw_weights(rng, m, in_shape, dtype) for m in models]
    if callable(lr):
        lr = lr(rng)
    h, w, c = in_shape
    if pixel == "normal":
        x = rng.standard_normal(size=(B, h, w, c)).astype(np.float32)
    else:
        x = rng.uniform(0.0, 1.0, size=(B, h, w, c)).astype(np.float32)
    if dtype == BF16:
        x = to_bf16_representable(x)
    labels = rng.integers(0, n_classes, size=B).astype(np.int32)
    return PackWorkload(name, dtype, B, in_shape, models, list(batch), weights,
                        np.asarray(lr, dtype=np.float32), x, labels, steps, n_classes, meta or {})


def mlp(widths: Sequence[int], n_classes: int) -> List[Layer]:
    layers: List[Layer] = []
    for wdt in widths:
        layers += [("linear", int(wdt)), ("relu",)]
    layers.append(("linear", int(n_classes)))
    return layers


def config1(seed: int = 0, K: int = 2, B: int = 32, D: int = 784, hidden: int = 128,
            n_classes: int = 10, lr=(0.01, 0.1)) -> PackWorkload:
    """K packed MLPs D-hidden-C, fp32, x ~ N(0,1), one step."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    models = [mlp([hidden], n_classes) for _ in range(K)]
    lr = [lr[k % len(lr)] for k in range(K)]
    return _finish("c1", F32, B, (1, 1, D), models, [B] * K, lr, rng, "normal", n_classes, 1)


def config2(seed: int = 1, K: int = 8, B: int = 256, D: int = 3072, hidden=(1024, 1024),
            n_classes: int = 10, steps: int = 10, dtype: str = BF16) -> PackWorkload:
    """K packed MLPs D-h-h-C, bf16 operands with fp32 accumulate and master, lr log-uniform."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    models = [mlp(hidden, n_classes) for _ in range(K)]
    lr = lambda r: 10.0 ** r.uniform(-4.0, -1.0, size=K)
    return _finish("c2", dtype, B, (1, 1, D), models, [B] * K, lr, rng, "normal", n_classes, steps)


def small_cnn(widths=(32, 64, 128), n_classes: int = 10) -> List[Layer]:
    """conv3x3(w0)-ReLU-conv3x3(w1)-ReLU-conv3x3(w2, stride 2)-ReLU-GAP-FC."""
    return [("conv3x3", widths[0], 1), ("relu",), ("conv3x3", widths[1], 1), ("relu",),
            ("conv3x3", widths[2], 2), ("relu",), ("gap",), ("linear", n_classes)]


def config3(seed: int = 2, K: int = 4, B: int = 128, size: int = 32, widths=(32, 64, 128),
            n_classes: int = 10, steps: int = 5, dtype: str = F32) -> PackWorkload:
    """K packed small CNNs on size x size x 3 images, fp32, pixels ~ U(0,1), lr = 10^U(-3,-1)."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    models = [small_cnn(widths, n_classes) for _ in range(K)]
    lr = lambda r: 10.0 ** r.uniform(-3.0, -1.0, size=K)
    return _finish("c3", dtype, B, (size, size, 3), models, [B] * K, lr, rng, "uniform", n_classes, steps)


def config4(seed: int = 3, K: int = 32, B: int = 128, D: int = 3072, n_classes: int = 10,
            width_choices=(64, 128, 256, 512, 1024), steps: int = 10, dtype: str = BF16) -> PackWorkload:
    """K heterogeneous MLPs: 2-4 hidden layers, widths drawn from `width_choices`, per-model
    learning rate 10^U(-4,-1) and batch scale in {1, 1/2, 1/4} (model k trains on the first b_k rows).
    Draw order per model: depth, widths, lr, batch scale."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    models, lr, batch = [], [], []
    for _ in range(K):
        depth = int(rng.integers(2, 5))
        widths = [int(width_choices[i]) for i in rng.integers(0, len(width_choices), size=depth)]
        lr.append(10.0 ** rng.uniform(-4.0, -1.0))
        scale = (1, 2, 4)[int(rng.integers(0, 3))]
        models.append(mlp(widths, n_classes))
        batch.append(max(1, B // scale))
    return _finish("c4", dtype, B, (1, 1, D), models, batch, lr, rng, "normal", n_classes, steps)


def resnet_style(widths=(64, 128, 256, 512), n_classes: int = 100) -> List[Layer]:
    """Stem conv3x3(w0)+ReLU, then one basic block per width (conv-ReLU-conv, add shortcut, ReLU),
    the first block at stride 1 and the others at stride 2; GAP; FC."""
    layers: List[Layer] = [("conv3x3", widths[0], 1), ("relu",)]
    for i, wdt in enumerate(widths):
        s = 1 if i == 0 else 2
        layers += [("res_begin",), ("conv3x3", wdt, s), ("relu",), ("conv3x3", wdt, 1), ("res_end",)]
    layers += [("gap",), ("linear", n_classes)]
    return layers


def config5(seed: int = 4, K: int = 4, B: int = 64, size: int = 64, widths=(64, 128, 256, 512),
            n_classes: int = 100, steps: int = 5, dtype: str = BF16) -> PackWorkload:
    """K packed ResNet-style CNNs on size x size x 3 images, bf16 operands, lr = 10^U(-3,-1.5)."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    models = [resnet_style(widths, n_classes) for _ in range(K)]
    lr = lambda r: 10.0 ** r.uniform(-3.0, -1.5, size=K)
    return _finish("c5", dtype, B, (size, size, 3), models, [B] * K, lr, rng, "uniform", n_classes, steps)


CONFIGS = {"c1": config1, "c2": config2, "c3": config3, "c4": config4, "c5": config5}


def custom(name: str, seed: int, dtype: str, B: int, in_shape, models, batch=None, lr=None,
           pixel: str = "normal", n_classes: int = 10, steps: int = 1) -> PackWorkload:
    """A workload from explicit layer lists (unit tests use it for small and odd shapes)."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    K = len(models)
    if lr is None:
        lr = lambda r: 10.0 ** r.uniform(-3.0, -1.0, size=K)
    return _finish(name, dtype, B, tuple(in_shape), [list(m) for m in models],
                   batch if batch is not None else [B] * K, lr, rng, pixel, n_classes, steps)


def labelled_dataset(seed: int, n: int, in_shape, dtype: str = F32, n_classes: int = 10):
    """n samples whose labels can be learnt: x ~ N(0, 1) and label = argmax of a fixed random linear
    map of x (a stand-in for the CIFAR-10 training set of the paper's search experiment, Section 5.3,
    with its 32x32x3 shape and 10 classes when called so).  Returns (x fp32 [n, H, W, C], labels int32 [n])."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    h, w, c = in_shape
    x = rng.standard_normal(size=(n, h, w, c)).astype(np.float32)
    if dtype == BF16:
        x = to_bf16_representable(x)
    teacher = rng.standard_normal(size=(h * w * c, n_classes)).astype(np.float32)
    labels = np.argmax(x.reshape(n, -1) @ teacher, axis=1).astype(np.int32)
    return x, labels
