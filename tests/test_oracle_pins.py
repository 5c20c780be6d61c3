"""Pins for the CPU oracle: it is checked against things other than itself - finite
differences, closed forms, brute-force definitions written out here, an independent autograd
library, and the paper's invariants (Section 2.2: a packed model trains exactly as if alone;
Section 3.1: pack is lossless and differentiable; Section 3.2: smaller batches are slices).
None of these tests needs a GPU."""
import math
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import pack_oracle as po

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = lambda s: np.random.default_rng(np.random.PCG64(s))


def _golden_pairs(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


# ----------------------------------------------------------------------------------------------
# bf16 rounding
# ----------------------------------------------------------------------------------------------

def test_q_bf16_hand_listed_bit_patterns():
    for src, want in _golden_pairs("bf16_rne.txt"):
        f = np.array([int(src, 16)], dtype=np.uint32).view(np.float32)
        got = po.q_bf16(f.astype(np.float64)).astype(np.float32).view(np.uint32)[0]
        assert got & 0xFFFF == 0
        assert (got >> 16) == int(want, 16), (src, hex(got >> 16), want)


def test_q_bf16_matches_library_conversion_on_random_fp32():
    r = RNG(11)
    a = (r.standard_normal(20000) * 10.0 ** r.uniform(-30, 30, 20000)).astype(np.float32)
    lib = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = po.q_bf16(a.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), lib.view(np.uint32))


def test_q_bf16_rounds_float64_once():
    # 1 + 2^-8 + 2^-40 is above the tie in float64 but rounds to the tie in float32.
    v = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert po.q_bf16(np.array([v]))[0] == 1.0 + 2.0 ** -7
    assert po.q_bf16(np.array([np.nan]))[0] != po.q_bf16(np.array([np.nan]))[0]


# ----------------------------------------------------------------------------------------------
# softmax cross-entropy
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("C,key", [(10, "ln10"), (100, "ln100")])
def test_xent_zero_logits_is_ln_C(C, key):
    gold = {k: float(v) for k, v in _golden_pairs("closed_forms.txt")}
    b = 7
    y = np.arange(b) % C
    loss, d, pred = po.softmax_xent(np.zeros((b, C)), y)
    assert abs(loss - gold[key]) < 1e-15 and abs(gold[key] - math.log(C)) < 1e-15
    want = np.full((b, C), 1.0 / C)
    want[np.arange(b), y] -= 1.0
    assert np.allclose(d, want / b, rtol=0, atol=1e-16)
    assert np.all(pred == 0)                       # ties resolve to the lowest index


def test_xent_invariants_and_brute_force():
    r = RNG(5)
    b, C = 9, 6
    z = r.standard_normal((b, C)) * 5
    y = r.integers(0, C, b)
    loss, d, pred = po.softmax_xent(z, y)
    # brute force, no max subtraction, python floats
    tot = 0.0
    for i in range(b):
        den = sum(math.exp(z[i, c]) for c in range(C))
        tot += -math.log(math.exp(z[i, y[i]]) / den)
        for c in range(C):
            p = math.exp(z[i, c]) / den
            assert abs(d[i, c] - (p - (1.0 if c == y[i] else 0.0)) / b) < 1e-14
    assert abs(loss - tot / b) < 1e-13
    assert np.allclose(d.sum(axis=1), 0.0, atol=1e-16)
    loss2, d2, pred2 = po.softmax_xent(z + 123.0, y)          # shift invariance
    assert abs(loss2 - loss) < 1e-12 and np.allclose(d2, d, atol=1e-14) and np.array_equal(pred, pred2)
    loss3, _, _ = po.softmax_xent(z * 1e3, y)                  # stability at large logits
    assert np.isfinite(loss3) and loss3 >= 0


def test_argmax_ties_lowest_index():
    z = np.array([[1.0, 3.0, 3.0, 2.0], [0.0, 0.0, 0.0, 0.0], [5.0, 1.0, 5.0, 5.0]])
    _, _, pred = po.softmax_xent(z, np.zeros(3, dtype=int))
    assert pred.tolist() == [1, 0, 0] and pred.dtype == np.int32


# ----------------------------------------------------------------------------------------------
# convolution against its definition
# ----------------------------------------------------------------------------------------------

def _conv_definition(x, W, bias, s):
    """Seven nested loops, straight from Z[b,i,j,o] = bias[o] + sum x[b,s*i+u-1,s*j+v-1,c] W[o,c,u,v]."""
    B, H, Wd, Cin = x.shape
    Co = W.shape[0]
    Ho, Wo = (H - 1) // s + 1, (Wd - 1) // s + 1
    z = np.zeros((B, Ho, Wo, Co))
    for b in range(B):
        for i in range(Ho):
            for j in range(Wo):
                for o in range(Co):
                    acc = bias[o]
                    for c in range(Cin):
                        for u in range(3):
                            for v in range(3):
                                yy, xx = s * i + u - 1, s * j + v - 1
                                if 0 <= yy < H and 0 <= xx < Wd:
                                    acc += x[b, yy, xx, c] * W[o, c, u, v]
                    z[b, i, j, o] = acc
    return z


@pytest.mark.parametrize("H,Wd,s", [(5, 4, 1), (6, 6, 2), (5, 7, 2), (1, 1, 1), (2, 2, 2)])
def test_conv_forward_equals_definition(H, Wd, s):
    r = RNG(H * 10 + Wd + s)
    x = r.standard_normal((2, H, Wd, 3))
    W = r.standard_normal((4, 3, 3, 3))
    b = r.standard_normal(4)
    assert np.allclose(po.conv3x3_forward(x, W, b, s), _conv_definition(x, W, b, s), rtol=0, atol=1e-13)


def test_conv_output_size_formula():
    for n in range(1, 12):
        assert po._conv_out(n, 1) == n
        assert po._conv_out(n, 2) == (n + 1) // 2
        assert wl.conv_out_size(n, 2) == po._conv_out(n, 2)


def test_conv_1x1_input_is_linear_on_centre_tap():
    r = RNG(3)
    x = r.standard_normal((5, 1, 1, 6))
    W = r.standard_normal((4, 6, 3, 3))
    b = r.standard_normal(4)
    z = po.conv3x3_forward(x, W, b, 1)
    assert np.allclose(z[:, 0, 0, :], x[:, 0, 0, :] @ W[:, :, 1, 1].T + b, atol=1e-14)


def test_conv_single_tap_is_shifted_copy():
    r = RNG(4)
    x = r.standard_normal((1, 5, 5, 1))
    for u in range(3):
        for v in range(3):
            W = np.zeros((1, 1, 3, 3))
            W[0, 0, u, v] = 1.0
            z = po.conv3x3_forward(x, W, np.zeros(1), 1)[0, :, :, 0]
            want = np.zeros((5, 5))
            for i in range(5):
                for j in range(5):
                    yy, xx = i + u - 1, j + v - 1
                    if 0 <= yy < 5 and 0 <= xx < 5:
                        want[i, j] = x[0, yy, xx, 0]
            assert np.array_equal(z, want)


@pytest.mark.parametrize("s", [1, 2])
def test_conv_backward_is_the_adjoint(s):
    r = RNG(20 + s)
    x = r.standard_normal((2, 6, 5, 3))
    W = r.standard_normal((4, 3, 3, 3))
    zero = np.zeros(4)
    z = po.conv3x3_forward(x, W, zero, s)
    y = r.standard_normal(z.shape)
    dW, db, dx = po.conv3x3_backward(x, W, s, y)
    assert abs(np.sum(z * y) - np.sum(x * dx)) < 1e-11          # <conv(x), y> = <x, conv^T(y)>
    assert abs(np.sum(z * y) - np.sum(W * dW)) < 1e-11          # conv is linear in W
    assert np.allclose(db, y.sum(axis=(0, 1, 2)))


def test_conv_matches_library_convolution():
    r = RNG(31)
    for s in (1, 2):
        x = r.standard_normal((3, 8, 6, 5))
        W = r.standard_normal((7, 5, 3, 3))
        b = r.standard_normal(7)
        want = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(W),
                                          torch.from_numpy(b), stride=s, padding=1).permute(0, 2, 3, 1).numpy()
        assert np.allclose(po.conv3x3_forward(x, W, b, s), want, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# pooling and shortcut
# ----------------------------------------------------------------------------------------------

def test_shortcut_is_a_fixed_linear_map_with_matching_adjoint():
    r = RNG(6)
    x = r.standard_normal((2, 6, 6, 3))
    out_shape = (2, 3, 3, 5)
    sc = po.shortcut_forward(x, out_shape)
    assert np.array_equal(sc[..., :3], x[:, ::2, ::2, :]) and np.all(sc[..., 3:] == 0)
    y = r.standard_normal(out_shape)
    assert abs(np.sum(sc * y) - np.sum(x * po.shortcut_backward(y, x.shape))) < 1e-12
    assert po.shortcut_forward(x, x.shape) is x


def test_gap_of_constant_and_zero_branch_block():
    layers = [("res_begin",), ("conv3x3", 3, 1), ("relu",), ("conv3x3", 3, 1), ("res_end",), ("gap",)]
    n = wl.num_params(layers, (4, 4, 3))
    net = po.Model(layers, (4, 4, 3), np.zeros(n))
    x = RNG(7).standard_normal((2, 4, 4, 3))
    logits, _ = net.forward(x)                          # zero branch: out = relu(shortcut(x))
    assert np.allclose(logits, np.maximum(x, 0).mean(axis=(1, 2)))
    net2 = po.Model([("gap",)], (4, 4, 3), np.zeros(0))
    assert np.allclose(net2.forward(np.full((2, 4, 4, 3), 2.5))[0], 2.5)


# ----------------------------------------------------------------------------------------------
# gradients: central finite differences and an independent autograd library
# ----------------------------------------------------------------------------------------------

NETS = {
    "mlp": ((1, 1, 5), wl.mlp([4], 3)),
    "mlp3": ((1, 1, 6), wl.mlp([5, 4, 4], 3)),
    "logreg": ((1, 1, 5), [("linear", 4)]),
    "cnn_s1s2": ((6, 6, 2), [("conv3x3", 3, 1), ("relu",), ("conv3x3", 4, 2), ("relu",), ("gap",), ("linear", 3)]),
    "cnn_odd": ((5, 7, 2), [("conv3x3", 3, 2), ("relu",), ("conv3x3", 3, 1), ("relu",), ("gap",), ("linear", 3)]),
    "res_identity": ((4, 4, 2), [("conv3x3", 3, 1), ("relu",), ("res_begin",), ("conv3x3", 3, 1), ("relu",),
                                 ("conv3x3", 3, 1), ("res_end",), ("gap",), ("linear", 3)]),
    "res_down": ((6, 6, 2), [("conv3x3", 3, 1), ("relu",), ("res_begin",), ("conv3x3", 5, 2), ("relu",),
                             ("conv3x3", 5, 1), ("res_end",), ("res_begin",), ("conv3x3", 5, 1), ("relu",),
                             ("conv3x3", 5, 1), ("res_end",), ("gap",), ("linear", 4)]),
    "conv_flatten_fc": ((3, 3, 2), [("conv3x3", 3, 1), ("relu",), ("linear", 3)]),
    # the other activations of the paper's search space (Table 3)
    "mlp_tanh": ((1, 1, 5), [("linear", 4), ("tanh",), ("linear", 4), ("tanh",), ("linear", 3)]),
    "mlp_sigmoid": ((1, 1, 5), [("linear", 4), ("sigmoid",), ("linear", 3)]),
    "mlp_leaky": ((1, 1, 6), [("linear", 5), ("leaky_relu",), ("linear", 4), ("leaky_relu",), ("linear", 3)]),
    "cnn_mixed_act": ((6, 6, 2), [("conv3x3", 3, 1), ("leaky_relu",), ("conv3x3", 4, 2), ("tanh",), ("gap",),
                                  ("linear", 4), ("sigmoid",), ("linear", 3)]),
}


def _make(name, seed, B=3):
    in_shape, layers = NETS[name]
    r = RNG(seed)
    n = wl.num_params(layers, in_shape)
    blob = r.standard_normal(n) * 0.7
    x = r.standard_normal((B,) + in_shape)
    C = po.Model(layers, in_shape, blob).n_classes
    y = r.integers(0, C, B)
    return in_shape, layers, blob, x, y


def _min_abs_preact(net, x):
    """Smallest |z| over all units that go through a ReLU mask (distance to the nearest kink)."""
    _, tape = net.forward(x)
    m = np.inf
    cur = np.asarray(x, dtype=np.float64)
    # recompute pre-activations layer by layer
    pi, res = 0, []
    for op in net.layers:
        if op[0] == "linear":
            W, b = net.params[pi]; pi += 1
            z = cur.reshape(cur.shape[0], -1) @ W.T + b
            cur = z.reshape(z.shape[0], 1, 1, -1)
        elif op[0] == "conv3x3":
            W, b = net.params[pi]; pi += 1
            cur = po.conv3x3_forward(cur, W, b, op[2])
        elif op[0] == "relu":
            m = min(m, np.abs(cur).min()); cur = np.maximum(cur, 0)
        elif op[0] == "leaky_relu":
            m = min(m, np.abs(cur).min()); cur = np.where(cur > 0, cur, po.LEAKY_SLOPE * cur)
        elif op[0] == "sigmoid":
            cur = 1.0 / (1.0 + np.exp(-cur))
        elif op[0] == "tanh":
            cur = np.tanh(cur)
        elif op[0] == "gap":
            cur = cur.mean(axis=(1, 2), keepdims=True)
        elif op[0] == "res_begin":
            res.append(cur)
        elif op[0] == "res_end":
            cur = cur + po.shortcut_forward(res.pop(), cur.shape)
            m = min(m, np.abs(cur).min()); cur = np.maximum(cur, 0)
    return m


@pytest.mark.parametrize("name", sorted(NETS))
def test_gradients_match_central_finite_differences(name):
    for seed in range(40):                              # pick data that stays away from ReLU kinks
        in_shape, layers, blob, x, y = _make(name, 100 + seed)
        if _min_abs_preact(po.Model(layers, in_shape, blob), x) > 1e-3:
            break
    else:
        pytest.fail("no kink-free sample found")
    net = po.Model(layers, in_shape, blob)
    _, _, grads = net.loss_and_grads(x, y)
    g = po.Model.flatten_grads(grads)
    h = 1e-6
    fd = np.zeros_like(blob)
    for i in range(blob.size):
        bp, bm = blob.copy(), blob.copy()
        bp[i] += h
        bm[i] -= h
        lp = po.Model(layers, in_shape, bp).loss_and_grads(x, y)[0]
        lm = po.Model(layers, in_shape, bm).loss_and_grads(x, y)[0]
        fd[i] = (lp - lm) / (2 * h)
    assert np.max(np.abs(fd - g)) <= 2e-7 * max(1.0, np.max(np.abs(g))), np.max(np.abs(fd - g))


def _torch_loss(layers, in_shape, blob_t, x, y):
    import torch.nn.functional as F
    cur = torch.from_numpy(x)
    off, res = 0, []
    h, w, c = in_shape
    for op in layers:
        if op[0] == "linear":
            fin = cur[0].numel()
            W = blob_t[off:off + op[1] * fin].reshape(op[1], fin); off += op[1] * fin
            b = blob_t[off:off + op[1]]; off += op[1]
            cur = F.linear(cur.reshape(cur.shape[0], -1), W, b).reshape(cur.shape[0], 1, 1, op[1])
        elif op[0] == "conv3x3":
            cin = cur.shape[3]
            n = op[1] * cin * 9
            W = blob_t[off:off + n].reshape(op[1], cin, 3, 3); off += n
            b = blob_t[off:off + op[1]]; off += op[1]
            cur = F.conv2d(cur.permute(0, 3, 1, 2), W, b, stride=op[2], padding=1).permute(0, 2, 3, 1)
        elif op[0] == "relu":
            cur = torch.relu(cur)
        elif op[0] == "leaky_relu":
            cur = F.leaky_relu(cur, negative_slope=0.2)
        elif op[0] == "sigmoid":
            cur = torch.sigmoid(cur)
        elif op[0] == "tanh":
            cur = torch.tanh(cur)
        elif op[0] == "gap":
            cur = cur.mean(dim=(1, 2), keepdim=True)
        elif op[0] == "res_begin":
            res.append(cur)
        elif op[0] == "res_end":
            src = res.pop()
            if src.shape != cur.shape:
                sub = src[:, ::2, ::2, :]
                src = F.pad(sub, (0, cur.shape[3] - sub.shape[3]))
            cur = torch.relu(cur + src)
    logits = cur.reshape(cur.shape[0], -1)
    return F.cross_entropy(logits, torch.from_numpy(np.asarray(y)).long(), reduction="mean"), logits


@pytest.mark.parametrize("name", sorted(NETS))
def test_gradients_match_independent_autograd(name):
    in_shape, layers, blob, x, y = _make(name, 7, B=4)
    bt = torch.from_numpy(blob.copy()).requires_grad_(True)
    loss_t, logits_t = _torch_loss(layers, in_shape, bt, x, y)
    loss_t.backward()
    net = po.Model(layers, in_shape, blob)
    loss, pred, grads = net.loss_and_grads(x, y)
    assert abs(loss - loss_t.item()) < 1e-12
    assert np.allclose(po.Model.flatten_grads(grads), bt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.array_equal(pred, logits_t.argmax(dim=1).numpy())


def test_full_size_layer_lists_match_independent_autograd_at_reduced_size():
    # The five benchmark architectures, shrunk, against the autograd library (one gradient each).
    cases = [wl.config1(B=4, D=20, hidden=8), wl.config2(B=4, D=24, hidden=(8, 8), K=2, dtype=wl.F32),
             wl.config3(B=2, size=6, widths=(3, 4, 5), K=1), wl.config4(B=8, D=16, K=3, width_choices=(4, 8), dtype=wl.F32),
             wl.config5(B=2, size=8, widths=(3, 4, 6, 8), K=1, n_classes=5, dtype=wl.F32)]
    for w in cases:
        for k in range(w.K):
            b = w.batch[k]
            x, y = w.x[:b].astype(np.float64), w.labels[:b]
            blob = w.weights[k].astype(np.float64)
            bt = torch.from_numpy(blob.copy()).requires_grad_(True)
            loss_t, _ = _torch_loss(w.models[k], w.in_shape, bt, x, y)
            loss_t.backward()
            loss, _, grads = po.Model(w.models[k], w.in_shape, blob).loss_and_grads(x, y)
            assert abs(loss - loss_t.item()) < 1e-11
            assert np.allclose(po.Model.flatten_grads(grads), bt.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_linear_only_model_is_multinomial_logistic_regression():
    in_shape, layers, blob, x, y = _make("logreg", 9, B=6)
    net = po.Model(layers, in_shape, blob)
    _, _, grads = net.loss_and_grads(x, y)
    X = x.reshape(6, -1)
    W, b = blob[:20].reshape(4, 5), blob[20:]
    Z = X @ W.T + b
    P = np.exp(Z) / np.exp(Z).sum(axis=1, keepdims=True)
    Y = np.eye(4)[y]
    assert np.allclose(grads[0][0], (P - Y).T @ X / 6, atol=1e-14)
    assert np.allclose(grads[0][1], (P - Y).sum(axis=0) / 6, atol=1e-14)


# ----------------------------------------------------------------------------------------------
# SGD step
# ----------------------------------------------------------------------------------------------

def test_sgd_is_linear_in_lr_and_zero_lr_is_identity():
    in_shape, layers, blob, x, y = _make("cnn_s1s2", 12)
    outs = []
    for lr in (0.0, 0.01, 0.3):
        net = po.Model(layers, in_shape, blob)
        loss, _, grads = net.sgd_step(x, y, lr)
        outs.append((net.blob(), po.Model.flatten_grads(grads), loss))
    assert np.array_equal(outs[0][0], blob)
    for lr, (w1, g, _) in zip((0.01, 0.3), outs[1:]):
        assert np.allclose((blob - w1) / lr, outs[0][1], rtol=1e-9, atol=1e-12)
    assert outs[0][2] == outs[1][2] == outs[2][2]           # reported loss is the pre-update loss


def test_loss_decreases_for_small_lr():
    in_shape, layers, blob, x, y = _make("mlp3", 13, B=8)
    net = po.Model(layers, in_shape, blob)
    l0 = net.sgd_step(x, y, 1e-3)[0]
    l1 = net.loss_and_grads(x, y)[0]
    assert l1 < l0


# ----------------------------------------------------------------------------------------------
# the paper's invariants
# ----------------------------------------------------------------------------------------------

class LiteralPackedMLP:
    """The packed network written out literally (Section 2.2: outputs concatenated; Section 3.4:
    one shared input): layer 1 is [W1^1 | ... | W1^K] on the shared input, deeper layers are
    dense block-diagonal matrices whose off-diagonal blocks are zero CONSTANTS, the output is the
    concatenation of all logits and the loss is the sum of the members' losses.  Written
    independently of the oracle's Model class; all members must have the same depth."""

    def __init__(self, widths_per_model, D, blobs, train_off_diagonal=False):
        self.K = len(widths_per_model)
        self.L = len(widths_per_model[0])
        self.train_off = train_off_diagonal
        self.Ws, self.bs, self.masks, self.col = [], [], [], []
        offs = [0] * self.K
        prev = None
        for l in range(self.L):
            outs = [w[l] for w in widths_per_model]
            ins = [D] * self.K if l == 0 else [w[l - 1] for w in widths_per_model]
            rows = sum(outs)
            cols = D if l == 0 else sum(ins)
            W = np.zeros((rows, cols)); M = np.zeros((rows, cols)); b = np.zeros(rows)
            r0 = c0 = 0
            for k in range(self.K):
                n = outs[k] * ins[k]
                Wk = blobs[k][offs[k]:offs[k] + n].reshape(outs[k], ins[k]); offs[k] += n
                bk = blobs[k][offs[k]:offs[k] + outs[k]]; offs[k] += outs[k]
                cs = slice(0, D) if l == 0 else slice(c0, c0 + ins[k])
                W[r0:r0 + outs[k], cs] = Wk; M[r0:r0 + outs[k], cs] = 1.0; b[r0:r0 + outs[k]] = bk
                r0 += outs[k]; c0 += ins[k]
            self.Ws.append(W); self.bs.append(b); self.masks.append(M); self.col.append(outs)

    def step(self, x, y, lr):
        K, L = self.K, self.L
        B = x.shape[0]
        acts = [x.reshape(B, -1)]
        for l in range(L):
            z = acts[-1] @ self.Ws[l].T + self.bs[l]
            acts.append(np.maximum(z, 0) if l < L - 1 else z)
        logits = acts[-1]
        d = np.zeros_like(logits)
        losses, c0 = [], 0
        for k in range(K):
            C = self.col[-1][k]
            zk = logits[:, c0:c0 + C]
            lse = np.log(np.exp(zk - zk.max(1, keepdims=True)).sum(1)) + zk.max(1)
            losses.append(np.mean(lse - zk[np.arange(B), y]))
            p = np.exp(zk - lse[:, None]); p[np.arange(B), y] -= 1
            d[:, c0:c0 + C] = p / B                        # gradient of the SUM of member losses
            c0 += C
        lr_rows = [np.concatenate([np.full(n, lr[k]) for k, n in enumerate(self.col[l])]) for l in range(L)]
        newW, newb = [], []
        for l in reversed(range(L)):
            dW = d.T @ acts[l]
            db = d.sum(0)
            if not self.train_off:
                dW = dW * self.masks[l]
            if l > 0:
                d = (d @ self.Ws[l]) * (acts[l] > 0)
            newW.append(self.Ws[l] - lr_rows[l][:, None] * dW); newb.append(self.bs[l] - lr_rows[l] * db)
        self.Ws, self.bs = newW[::-1], newb[::-1]
        return np.array(losses)

    def member_blob(self, k):
        parts = []
        for l in range(self.L):
            r0 = sum(self.col[l][:k]); r1 = r0 + self.col[l][k]
            if l == 0:
                Wk = self.Ws[l][r0:r1, :]
            else:
                c0 = sum(self.col[l - 1][:k]); Wk = self.Ws[l][r0:r1, c0:c0 + self.col[l - 1][k]]
            parts += [Wk.ravel(), self.bs[l][r0:r1]]
        return np.concatenate(parts)


def _hetero_mlps(seed, K=3, D=7, B=5, C=4):
    r = RNG(seed)
    widths = [[int(r.integers(3, 7)), int(r.integers(3, 7)), C] for _ in range(K)]
    models = [wl.mlp(w[:-1], C) for w in widths]
    blobs = [r.standard_normal(wl.num_params(m, (1, 1, D))) * 0.5 for m in models]
    x = r.standard_normal((B, 1, 1, D)); y = r.integers(0, C, B)
    lr = 10.0 ** r.uniform(-2, -0.5, K)
    return widths, models, blobs, x, y, lr


def test_packed_step_equals_K_independent_steps_literal_network():
    widths, models, blobs, x, y, lr = _hetero_mlps(21)
    D, B = 7, 5
    lit = LiteralPackedMLP(widths, D, blobs)
    ref = po.train_pack(models, (1, 1, D), blobs, [B] * 3, lr, x, y, steps=3)
    for t in range(3):
        losses = lit.step(x, y, lr)
        assert np.allclose(losses, ref["loss"][t], rtol=1e-12, atol=1e-13)
    for k in range(3):
        assert np.allclose(lit.member_blob(k), ref["blobs"][k], rtol=1e-12, atol=1e-13)
    # negative control: if the zero blocks were parameters they would pick up gradient and the
    # members would no longer train as if alone
    bad = LiteralPackedMLP(widths, D, blobs, train_off_diagonal=True)
    for t in range(3):
        bad_losses = bad.step(x, y, lr)
    assert not np.allclose(bad_losses, ref["loss"][2], rtol=1e-6)


def test_packing_order_is_irrelevant():
    widths, models, blobs, x, y, lr = _hetero_mlps(22, K=4)
    ref = po.train_pack(models, (1, 1, 7), blobs, [5, 3, 5, 2], lr, x, y, steps=2)
    perm = [2, 0, 3, 1]
    out = po.train_pack([models[i] for i in perm], (1, 1, 7), [blobs[i] for i in perm],
                        [[5, 3, 5, 2][i] for i in perm], lr[perm], x, y, steps=2)
    for j, i in enumerate(perm):
        assert np.array_equal(out["blobs"][j], ref["blobs"][i])
        assert np.array_equal(out["loss"][:, j], ref["loss"][:, i])
        assert np.array_equal(out["pred"][1][j], ref["pred"][1][i])


def test_member_is_independent_of_other_members_hyperparameters():
    widths, models, blobs, x, y, lr = _hetero_mlps(23)
    a = po.train_pack(models, (1, 1, 7), blobs, [5] * 3, lr, x, y, steps=2)
    lr2 = lr.copy(); lr2[1] *= 7.0
    b = po.train_pack(models, (1, 1, 7), blobs, [5] * 3, lr2, x, y, steps=2)
    assert np.array_equal(a["blobs"][0], b["blobs"][0]) and np.array_equal(a["blobs"][2], b["blobs"][2])
    assert not np.array_equal(a["blobs"][1], b["blobs"][1])


def test_smaller_batch_is_a_prefix_slice():
    widths, models, blobs, x, y, lr = _hetero_mlps(24)
    xb = x.copy(); xb[3:] = np.nan                       # rows >= b_k must never be touched
    out = po.train_pack(models[:1], (1, 1, 7), blobs[:1], [3], lr[:1], xb, y, steps=2)
    alone = po.Model(models[0], (1, 1, 7), blobs[0])
    for _ in range(2):
        alone.sgd_step(x[:3], y[:3], float(lr[0]))
    assert np.array_equal(out["blobs"][0], alone.blob()) and np.all(np.isfinite(out["blobs"][0]))
    assert len(out["pred"][0][0]) == 3


def test_singleton_pack_is_an_ordinary_trainer():
    in_shape, layers, blob, x, y = _make("res_down", 31, B=4)
    out = po.train_pack([layers], in_shape, [blob], [4], [0.05], x, y, steps=2, keep_grads=True)
    bt = torch.from_numpy(blob.copy()).requires_grad_(True)
    for t in range(2):
        loss_t, _ = _torch_loss(layers, in_shape, bt, x, y)
        g, = torch.autograd.grad(loss_t, bt)
        assert abs(loss_t.item() - out["loss"][t, 0]) < 1e-12
        assert np.allclose(g.numpy(), out["grads"][t][0], rtol=1e-9, atol=1e-12)
        bt = (bt - 0.05 * g).detach().requires_grad_(True)
    assert np.allclose(bt.detach().numpy(), out["blobs"][0], rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------------------------
# rounded (bf16) mode
# ----------------------------------------------------------------------------------------------

def test_rounded_mode_is_close_to_exact_and_stores_bf16_operands():
    w = wl.config2(B=16, D=64, hidden=(32, 32), K=2)
    blob = w.weights[0].astype(np.float64)
    x, y = w.x.astype(np.float64), w.labels
    ex = po.Model(w.models[0], w.in_shape, blob, "exact").loss_and_grads(x, y)
    rd = po.Model(w.models[0], w.in_shape, blob, "rounded")
    lr_, _, gr = rd.loss_and_grads(x, y)
    ge, gr = po.Model.flatten_grads(ex[2]), po.Model.flatten_grads(gr)
    assert abs(lr_ - ex[0]) < 2e-2 * abs(ex[0])
    assert np.linalg.norm(gr - ge) < 2e-2 * np.linalg.norm(ge)
    assert not np.array_equal(gr, ge)
    _, tape = rd.forward(x)
    for rec in tape:
        if rec[0] == "relu":
            assert np.array_equal(po.q_bf16(rec[1]), rec[1])


def test_weight_rounding_mode_equals_exact_while_weights_are_representable_then_lags():
    # With bf16-representable initial weights the first step of "weights" mode IS the exact step;
    # after the update the master is no longer representable and the operand copy lags behind it.
    w = wl.config2(B=16, D=64, hidden=(32, 32), K=1)
    args = (w.models, w.in_shape, [w.weights[0].astype(np.float64)], w.batch, [0.05], w.x.astype(np.float64), w.labels)
    ex = po.train_pack(*args, steps=3, mode="exact", keep_grads=True)
    wt = po.train_pack(*args, steps=3, mode="weights", keep_grads=True)
    assert ex["loss"][0, 0] == wt["loss"][0, 0] and np.array_equal(ex["grads"][0][0], wt["grads"][0][0])
    assert ex["loss"][1, 0] != wt["loss"][1, 0]
    assert abs(ex["loss"][2, 0] - wt["loss"][2, 0]) < 0.05 * ex["loss"][2, 0]


def _bf16_by_hand(v):
    """Round one Python float to bfloat16 (8 significant bits, halves to even) with integer rounding of
    the scaled significand; written here so that the pin below does not lean on the oracle's q_bf16."""
    if v == 0.0:
        return 0.0
    m, e = math.frexp(v)                 # v = m * 2**e, 0.5 <= |m| < 1
    return math.ldexp(round(m * 256.0), e - 8)   # round() rounds halves to even; m * 256 is exact


def _residual_fork_by_hand(drop=()):
    """One training example through   conv - relu - [ conv - relu - conv ] + shortcut - relu - gap - linear(2)
    on a 1 x 2 image with one channel, every convolution with only its centre tap non-zero, so that each
    pixel is a chain of scalar operations that can be followed by hand.  `r(i, v)` is rounding point
    number i of the bf16 configuration: the per-step operand copy of each weight (1-4), every stored
    activation (5-8: first relu, inner relu, block output, pooled value) and every stored gradient
    (9: dlogits, 10: gradient wrt the pooled value, 11: after the inner relu's mask, 12: THE FORK, the
    sum of the branch's and the shortcut's gradient, 13: after the first relu's mask, which for a
    0 / 1 mask is the same store as 12).  Points in `drop`
    are skipped, which is how the test shows that each of them is pinned."""
    def r(i, v):
        return v if i in drop else _bf16_by_hand(v)

    xa, xb = 0.8125, 1.40625                                  # bf16-representable data
    w1, b1, w2, b2, w3, b3 = 0.7431, 0.10001, 0.611, 0.3, 0.9017, -0.05
    W4, b4, label = (0.37, -0.83), (0.01, -0.02), 1
    q1, q2, q3 = r(1, w1), r(2, w2), r(3, w3)
    q4 = (r(4, W4[0]), r(4, W4[1]))
    # forward, pixel by pixel
    h1 = [r(5, max(x * q1 + b1, 0.0)) for x in (xa, xb)]
    h2 = [r(6, max(h * q2 + b2, 0.0)) for h in h1]
    h3 = [r(7, max(h2[j] * q3 + b3 + h1[j], 0.0)) for j in range(2)]
    pooled = r(8, (h3[0] + h3[1]) / 2.0)
    logits = [pooled * q4[c] + b4[c] for c in range(2)]
    mx = max(logits)
    ex = [math.exp(z - mx) for z in logits]
    loss = mx + math.log(ex[0] + ex[1]) - logits[label]
    # backward
    dz = [r(9, ex[c] / (ex[0] + ex[1]) - (1.0 if c == label else 0.0)) for c in range(2)]
    dW4 = [dz[c] * pooled for c in range(2)]
    g_pool = r(10, dz[0] * q4[0] + dz[1] * q4[1])
    g3 = [g_pool / 2.0 * (1.0 if h3[j] > 0 else 0.0) for j in range(2)]          # exact in bf16: halving
    g2 = [r(11, g3[j] * q3 * (1.0 if h2[j] > 0 else 0.0)) for j in range(2)]
    fork = [r(12, g2[j] * q2 + g3[j]) for j in range(2)]
    g1 = [r(13, fork[j] * (1.0 if h1[j] > 0 else 0.0)) for j in range(2)]

    def conv_dw(d, inp):
        # [3][3] taps of a one-row image: row u = 1 only; tap v reads pixel j + v - 1
        return {"centre": d[0] * inp[0] + d[1] * inp[1], "left": d[1] * inp[0], "right": d[0] * inp[1], "bias": d[0] + d[1]}

    return {"loss": loss, "dW1": conv_dw(g1, (xa, xb)), "dW2": conv_dw(g2, h1), "dW3": conv_dw(g3, h2),
            "dW4": dW4, "db4": dz}


def test_rounded_mode_rounds_exactly_where_the_configuration_says_hand_worked_residual_fork():
    """The oracle's mode "rounded" against a residual block worked by hand (the scalar chain above, with
    its own bf16 rounding): every gradient must agree to float64 rounding.  Leaving out any single
    rounding point in the hand computation (the fork included) moves at least one gradient far beyond
    that, so a q() dropped from, or added to, the oracle at any of those places fails this test."""
    for src, want in _golden_pairs("bf16_rne.txt"):          # the hand rounding itself, on the listed bit patterns
        f = float(np.array([int(src, 16)], dtype=np.uint32).view(np.float32)[0])
        if math.isfinite(f) and 1e-30 < abs(f) < 1e38:
            got = np.array([_bf16_by_hand(f)], dtype=np.float32).view(np.uint32)[0]
            assert got & 0xFFFF == 0 and (got >> 16) == int(want, 16), src
    layers = [("conv3x3", 1, 1), ("relu",), ("res_begin",), ("conv3x3", 1, 1), ("relu",), ("conv3x3", 1, 1), ("res_end",),
              ("gap",), ("linear", 2)]
    centre = lambda w: [0, 0, 0, 0, w, 0, 0, 0, 0]
    blob = np.array(centre(0.7431) + [0.10001] + centre(0.611) + [0.3] + centre(0.9017) + [-0.05]
                    + [0.37, -0.83] + [0.01, -0.02])
    x = np.array([0.8125, 1.40625]).reshape(1, 1, 2, 1)
    net = po.Model(layers, (1, 2, 1), blob, "rounded")
    loss, pred, grads = net.loss_and_grads(x, np.array([1]))

    def flat(h):
        out = []
        for name in ("dW1", "dW2", "dW3"):
            d = h[name]
            out += [0, 0, 0, d["left"], d["centre"], d["right"], 0, 0, 0, d["bias"]]
        return np.array(out + h["dW4"] + h["db4"])

    got = po.Model.flatten_grads(grads)
    want = _residual_fork_by_hand()
    assert abs(loss - want["loss"]) <= 1e-14 * abs(want["loss"])
    assert np.allclose(got, flat(want), rtol=1e-13, atol=0)
    assert np.all(flat(want)[[3, 4, 5, 9, 13, 14, 15, 19, 23, 24, 25, 29, 30, 31, 32, 33]] != 0)   # every checked entry is live
    # 12 and 13 are one store when the mask between them is 0 / 1 (rounding twice changes nothing), so
    # they are dropped together; alone, either must leave the result as it is
    for alone in (12, 13):
        assert np.array_equal(flat(_residual_fork_by_hand(drop=(alone,))), flat(want))
    for point in [(i,) for i in range(1, 12)] + [(12, 13)]:
        other = _residual_fork_by_hand(drop=point)
        moved = max(np.max(np.abs(flat(other) - flat(want)) / np.maximum(np.abs(flat(want)), 1e-300)),
                    abs(other["loss"] - want["loss"]) / abs(want["loss"]))
        assert moved > 1e-6, f"rounding point {point} is not pinned by this example (moves the result by {moved})"
        assert not np.allclose(got, flat(other), rtol=1e-9, atol=0) or abs(loss - other["loss"]) > 1e-9 * abs(loss), point
