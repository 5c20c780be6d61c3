"""CPU oracle for packed training.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
import, call or link this file; it exists so that tests, the smoke check and the bench's CPU
baseline leg have a slow, plain, independent statement of what a packed step must produce.

What it computes.  `pack` (paper Section 2.2 and 3.1) joins K networks into one by concatenating
their outputs; the operation is lossless, so input, output and back-propagation of every member
are those of the member trained alone (the isolation guarantee of Section 2.2).  With a shared
dataset the K inputs collapse into one input (Section 3.4), members with a smaller batch size
train on a slice of the shared batch (Section 3.2), every member carries its own
hyper-parameters (Section 2.2, trait (a)), and all members are differentiated and updated in one
synchronised step (Section 2.2).  Because the result has this plain definition, the oracle IS
that definition: it trains each of the K models SEPARATELY, one ordinary mini-batch SGD step at
a time, in float64, on rows [0, b_k) of the shared batch.

The paper fixes none of the layer numerics; the readings used here are:
  * loss = mean over the model's own b_k rows of softmax cross-entropy (max-subtracted
    log-sum-exp); the packed loss is the unweighted sum over models, so each model's gradient is
    the gradient of its own loss;
  * plain SGD, W <- W - lr_k * dW, all parameters of a step updated from gradients taken at the
    pre-update weights; the reported loss is the pre-update loss;
  * every linear / conv layer has a bias; conv is 3x3, zero padding 1, stride 1 or 2;
  * ReLU derivative is 0 at 0 (mask z > 0, taken after the bias add);
  * the other activations of the paper's search space (Table 3): sigmoid 1/(1+e^-z), tanh, and
    leaky ReLU max(z, a*z) with a = 0.2 (the default slope of the framework the paper ran on;
    the paper names no slope); derivative of leaky ReLU at 0 is a;
  * the other optimisers of Table 3, each with its state kept beside the model (Section 2.2), all
    applied to gradients taken at the pre-update weights:
      momentum  acc <- mu*acc + g;  W <- W - lr*acc                       (acc starts at 0)
      adagrad   acc <- acc + g*g;   W <- W - lr*g/sqrt(acc)               (acc starts at acc0 > 0)
      adam      m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g*g;  t <- t+1;
                W <- W - lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)      (m, v, t start at 0)
    The paper prints no update formula; these are the published definitions of the methods it
    names (heavy-ball momentum; Duchi et al. without damping term; Kingma & Ba, Algorithm 1);
  * residual block: y = relu(branch(x) + shortcut(x)); the shortcut is the identity when shapes
    agree, otherwise the parameter-free form sc[b,i,j,c] = x[b,2i,2j,c] for c < Cin, 0 above;
  * argmax returns the smallest index attaining the maximum;
  * a linear layer applied to an image flattens it in NHWC order.

bf16 packs ("bf16 inputs/weights, fp32 accumulate, fp32 master weights") have three modes here:
  mode "exact"   - float64 throughout; only the data (x, initial weights) is bf16-representable.
                   Equals the other modes' definition at step 1 up to activation rounding.
  mode "weights" - the precision the configuration itself fixes: every step multiplies by
                   q(W_master), the bf16 copy of the master weights, and updates the unrounded
                   master; everything else float64.  This is the reference for losses and
                   weights of bf16 packs (an update smaller than half a bf16 ulp of a weight is
                   invisible to the next forward pass until it accumulates in the master, so
                   from step 2 on this differs from "exact" by far more than any tolerance).
  mode "rounded" - "weights" plus q() = round-to-nearest-even to bf16 applied where the
                   device stores a matrix-core operand: the per-step operand copy of each weight
                   tensor (biases stay fp32), every stored activation (post-ReLU / post-residual,
                   GAP output; logits stay unrounded), every stored gradient with respect to a
                   layer output (after the ReLU / residual mask, after the sum at a residual
                   fork, and before any layer that reads it as an operand, dlogits included).

Parity status of the pieces: gradients of every layer type are pinned by central finite
differences, by a dense block-diagonal "literal packed network" formulation, by closed forms
(ln C loss, logistic regression) and by an independent autograd library on small shapes (see
tests/test_oracle_*.py).  The specific architecture readings (conv stride placement in the
small CNN, the residual shortcut form, the heterogeneous-MLP sampling recipe, the
initialisation) are choices the paper does not make: parity unpinned for those, both sides
simply follow the same written reading.
"""
from __future__ import annotations

import numpy as np

__all__ = ["q_bf16", "Model", "train_pack", "softmax_xent", "apply_update", "new_opt_state", "LEAKY_SLOPE"]

LEAKY_SLOPE = 0.2


def q_bf16(a):
    """Round float64 values to the nearest bfloat16 (8-bit significand, ties to even), directly
    from float64 so that no double rounding through float32 occurs.  Infinities and NaN pass
    through; magnitudes beyond the largest finite bf16 become infinite; below 2^-126 the spacing
    is the subnormal 2^-133."""
    a = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(a)                      # a = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                 # subnormal range keeps a fixed quantum
    quantum = np.ldexp(1.0, e - 8)
    with np.errstate(invalid="ignore", over="ignore"):
        r = np.rint(a / quantum) * quantum  # rint rounds halves to even
    big = np.ldexp(2.0 - 2.0 ** -7, 127)    # largest finite bf16
    r = np.where(np.abs(r) > big, np.copysign(np.inf, r), r)
    return np.where(np.isfinite(a), r, a)


def _ident(a):
    return a


def softmax_xent(logits, y):
    """Mean softmax cross-entropy over rows, its gradient with respect to the logits, and the
    argmax (lowest index on ties).  logits [b, C] float64, y [b] integer labels."""
    b = logits.shape[0]
    m = logits.max(axis=1, keepdims=True)
    ex = np.exp(logits - m)
    s = ex.sum(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(s[:, 0])
    loss = np.sum(lse - logits[np.arange(b), y]) / b
    p = ex / s
    p[np.arange(b), y] -= 1.0
    return loss, p / b, np.argmax(logits, axis=1).astype(np.int32)


def _act_forward(kind, z):
    if kind == "relu":
        return np.maximum(z, 0.0)
    if kind == "leaky_relu":
        return np.where(z > 0.0, z, LEAKY_SLOPE * z)
    if kind == "sigmoid":
        return 1.0 / (1.0 + np.exp(-z))
    if kind == "tanh":
        return np.tanh(z)
    raise ValueError(kind)


def _act_derivative(kind, out):
    """f'(z) written in terms of the stored output out = f(z)."""
    if kind == "relu":
        return (out > 0.0).astype(np.float64)
    if kind == "leaky_relu":
        return np.where(out > 0.0, 1.0, LEAKY_SLOPE)
    if kind == "sigmoid":
        return out * (1.0 - out)
    if kind == "tanh":
        return 1.0 - out * out
    raise ValueError(kind)


ACTIVATIONS = ("relu", "leaky_relu", "sigmoid", "tanh")


def new_opt_state(opt, shape):
    """Fresh optimiser state for one parameter tensor: a list of arrays (possibly empty)."""
    kind = opt["kind"]
    if kind == "sgd":
        return []
    if kind == "momentum":
        return [np.zeros(shape)]
    if kind == "adagrad":
        return [np.full(shape, float(opt.get("acc0", 0.1)))]
    if kind == "adam":
        return [np.zeros(shape), np.zeros(shape)]
    raise ValueError(kind)


def apply_update(opt, w, g, state, lr, t):
    """One optimiser step on one tensor, in place.  `t` is the number of this step (1 for the
    first); `state` comes from new_opt_state.  Formulas as listed in the module header."""
    kind = opt["kind"]
    if kind == "sgd":
        w -= lr * g
    elif kind == "momentum":
        acc, = state
        acc *= float(opt.get("mu", 0.9))
        acc += g
        w -= lr * acc
    elif kind == "adagrad":
        acc, = state
        acc += g * g
        w -= lr * g / np.sqrt(acc)
    elif kind == "adam":
        m, v = state
        b1, b2, eps = float(opt.get("beta1", 0.9)), float(opt.get("beta2", 0.999)), float(opt.get("eps", 1e-8))
        m *= b1
        m += (1.0 - b1) * g
        v *= b2
        v += (1.0 - b2) * g * g
        mhat = m / (1.0 - b1 ** t)
        vhat = v / (1.0 - b2 ** t)
        w -= lr * mhat / (np.sqrt(vhat) + eps)
    else:
        raise ValueError(kind)


def _conv_out(n, s):
    return (n + 2 - 3) // s + 1


def conv3x3_forward(x, W, bias, s):
    """Z[b,i,j,o] = bias[o] + sum_{c,u,v} xpad[b, s*i+u, s*j+v, c] * W[o,c,u,v], xpad = x with one
    ring of zeros.  x is [b,H,W,Cin] (NHWC), W is [Cout,Cin,3,3]."""
    b, H, Wd, _ = x.shape
    Ho, Wo = _conv_out(H, s), _conv_out(Wd, s)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    z = np.broadcast_to(bias, (b, Ho, Wo, W.shape[0])).copy()
    for u in range(3):
        for v in range(3):
            patch = xp[:, u:u + s * (Ho - 1) + 1:s, v:v + s * (Wo - 1) + 1:s, :]
            z += patch @ W[:, :, u, v].T
    return z


def conv3x3_backward(x, W, s, dz, need_dx=True):
    """Adjoint of conv3x3_forward: gradients with respect to W, bias and (optionally) x."""
    b, H, Wd, Cin = x.shape
    Ho, Wo = dz.shape[1], dz.shape[2]
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    dW = np.zeros_like(W)
    dxp = np.zeros_like(xp) if need_dx else None
    dz2 = dz.reshape(-1, dz.shape[3])
    for u in range(3):
        for v in range(3):
            rows = slice(u, u + s * (Ho - 1) + 1, s)
            cols = slice(v, v + s * (Wo - 1) + 1, s)
            patch = xp[:, rows, cols, :].reshape(-1, Cin)
            dW[:, :, u, v] = dz2.T @ patch
            if need_dx:
                dxp[:, rows, cols, :] += dz @ W[:, :, u, v]
    db = dz2.sum(axis=0)
    dx = dxp[:, 1:H + 1, 1:Wd + 1, :] if need_dx else None
    return dW, db, dx


def shortcut_forward(x, out_shape):
    """Parameter-free shortcut of a residual block: identity when shapes agree, otherwise
    subsample every second pixel and pad the new channels with zeros."""
    if x.shape == out_shape:
        return x
    _, Ho, Wo, Co = out_shape
    sc = np.zeros(out_shape, dtype=x.dtype)
    sub = x[:, ::2, ::2, :]
    assert sub.shape[1] == Ho and sub.shape[2] == Wo and x.shape[3] <= Co, "shortcut shape"
    sc[..., :x.shape[3]] = sub
    return sc


def shortcut_backward(dsc, x_shape):
    if dsc.shape == x_shape:
        return dsc
    dx = np.zeros(x_shape, dtype=dsc.dtype)
    dx[:, ::2, ::2, :] = dsc[..., :x_shape[3]]
    return dx


class Model:
    """One network trained alone.  `layers` is a list of tuples ("linear", out),
    ("conv3x3", out, stride), ("relu",) / ("leaky_relu",) / ("sigmoid",) / ("tanh",), ("gap",),
    ("res_begin",), ("res_end",); `blob` is the flat weight vector (linear W[out][in], b[out];
    conv W[Cout][Cin][3][3], b[Cout]).  `opt` is the optimiser: {"kind": "sgd"} (default),
    {"kind": "momentum", "mu": 0.9}, {"kind": "adagrad", "acc0": 0.1} or
    {"kind": "adam", "beta1": 0.9, "beta2": 0.999, "eps": 1e-8}."""

    def __init__(self, layers, in_shape, blob, mode="exact", acc_noise=None, opt=None):
        """`acc_noise`, if given, is a function applied to every matrix-product result a device
        would hold in an fp32 accumulator (forward pre-activations, input gradients) before
        anything else looks at it.  It is a sensitivity probe for tests - how far do the results
        move when those sums carry accumulation-order noise - and is the identity by default."""
        assert mode in ("exact", "weights", "rounded")
        self.acc = acc_noise if acc_noise is not None else _ident
        self.layers = [tuple(op) for op in layers]
        self.in_shape = tuple(in_shape)
        self.q = q_bf16 if mode == "rounded" else _ident          # stored activations / gradients
        self.qw = q_bf16 if mode in ("weights", "rounded") else _ident   # per-step operand copy of W
        self.params = []                                  # [W, b] per parameterised layer
        blob = np.asarray(blob, dtype=np.float64)
        h, w, c = self.in_shape
        off = 0
        for op in self.layers:
            if op[0] == "linear":
                shp = (op[1], h * w * c)
                h, w, c = 1, 1, op[1]
            elif op[0] == "conv3x3":
                shp = (op[1], c, 3, 3)
                h, w, c = _conv_out(h, op[2]), _conv_out(w, op[2]), op[1]
            else:
                if op[0] == "gap":
                    h, w = 1, 1
                continue
            n = int(np.prod(shp))
            W = blob[off:off + n].reshape(shp).copy()
            b = blob[off + n:off + n + shp[0]].copy()
            off += n + shp[0]
            self.params.append([W, b])
        assert off == blob.size, "weight blob does not match the layer list"
        self.n_classes = c
        self.opt = dict(opt) if opt is not None else {"kind": "sgd"}
        self.opt_state = [[new_opt_state(self.opt, W.shape), new_opt_state(self.opt, b.shape)] for W, b in self.params]
        self.t = 0

    # -- flat views ---------------------------------------------------------------------------
    def blob(self):
        return np.concatenate([np.concatenate([W.ravel(), b.ravel()]) for W, b in self.params])

    @staticmethod
    def flatten_grads(grads):
        return np.concatenate([np.concatenate([dW.ravel(), db.ravel()]) for dW, db in grads])

    # -- forward ------------------------------------------------------------------------------
    def forward(self, X):
        """Returns logits [b, C] and the tape needed by backward.  X is [b, H, W, C]."""
        q = self.q
        cur = np.asarray(X, dtype=np.float64)
        tape, pi, res_src = [], 0, []
        for idx, op in enumerate(self.layers):
            kind = op[0]
            if kind == "linear":
                W, b = self.params[pi]
                cur = q(cur)                       # a stored operand is a rounded operand
                flat = cur.reshape(cur.shape[0], -1)
                z = self.acc(flat @ self.qw(W).T) + b
                tape.append(("linear", pi, cur))
                cur = z.reshape(z.shape[0], 1, 1, z.shape[1])
                pi += 1
            elif kind == "conv3x3":
                W, b = self.params[pi]
                cur = q(cur)
                z = self.acc(conv3x3_forward(cur, self.qw(W), np.zeros_like(b), op[2])) + b
                tape.append(("conv3x3", pi, cur, op[2]))
                cur = z
                pi += 1
            elif kind in ACTIVATIONS:
                cur = q(_act_forward(kind, cur))
                tape.append((kind, cur))
            elif kind == "gap":
                cur = q(cur)
                tape.append(("gap", cur.shape))
                cur = q(cur.mean(axis=(1, 2), keepdims=True))
            elif kind == "res_begin":
                cur = q(cur)
                res_src.append(cur)
                tape.append(("res_begin",))
            elif kind == "res_end":
                src = res_src.pop()
                cur = q(np.maximum(cur + shortcut_forward(src, cur.shape), 0.0))
                tape.append(("res_end", cur, src.shape))
            else:
                raise ValueError(op)
        assert not res_src, "res_begin without res_end"
        logits = cur.reshape(cur.shape[0], -1)
        return logits, tape

    # -- backward -----------------------------------------------------------------------------
    def loss_and_grads(self, X, y):
        """loss (mean over rows), argmax predictions, and [dW, db] per parameterised layer."""
        q = self.q
        logits, tape = self.forward(X)
        self.last_logits = logits                  # kept for tests that compare the argmax margin
        loss, dlogits, pred = softmax_xent(logits, np.asarray(y))
        g = dlogits.reshape(dlogits.shape[0], 1, 1, -1)
        grads = [None] * len(self.params)
        pending = []                               # shortcut gradients waiting for res_begin
        first_param = 0
        # Rounding rule of the "rounded" mode: a gradient is rounded when it is stored, and it is
        # stored (a) after a ReLU / residual mask, (b) after the sum at a residual fork, and
        # (c) before any layer that reads it as an operand.  Products are formed from rounded
        # operands and accumulate unrounded.
        for rec in reversed(tape):
            kind = rec[0]
            if g is None:                          # everything left is upstream of the first
                break                              # parameterised layer: its input is data
            if kind == "linear":
                _, pi, inp = rec
                W, _b = self.params[pi]
                dz = q(g).reshape(g.shape[0], -1)
                flat = inp.reshape(inp.shape[0], -1)
                grads[pi] = [dz.T @ flat, dz.sum(axis=0)]
                g = self.acc(dz @ self.qw(W)).reshape(inp.shape) if pi != first_param else None
            elif kind == "conv3x3":
                _, pi, inp, s = rec
                W, _b = self.params[pi]
                dW, db, dx = conv3x3_backward(inp, self.qw(W), s, q(g), need_dx=(pi != first_param))
                grads[pi] = [dW, db]
                g = self.acc(dx) if dx is not None else None
            elif kind in ACTIVATIONS:
                g = q(g * _act_derivative(kind, rec[1]))
            elif kind == "gap":
                shp = rec[1]
                g = np.broadcast_to(q(g) / (shp[1] * shp[2]), shp).copy()
            elif kind == "res_end":
                _, out, src_shape = rec
                g = q(g * (out > 0.0))
                pending.append(shortcut_backward(g, src_shape))
            elif kind == "res_begin":
                g = q(g + pending.pop())
        return loss, pred, grads

    def sgd_step(self, X, y, lr):
        """One training step with the model's optimiser (plain mini-batch SGD unless `opt` says
        otherwise); returns (pre-update loss, predictions, grads)."""
        loss, pred, grads = self.loss_and_grads(X, y)
        self.t += 1
        for (W, b), (dW, db), (sW, sb) in zip(self.params, grads, self.opt_state):
            apply_update(self.opt, W, dW, sW, lr, self.t)
            apply_update(self.opt, b, db, sb, lr, self.t)
        return loss, pred, grads

    def opt_state_blob(self, slot):
        """State array `slot` (0 or 1) of every tensor, flattened in the blob layout."""
        return np.concatenate([np.concatenate([sW[slot].ravel(), sb[slot].ravel()]) for sW, sb in self.opt_state])


def train_pack(models, in_shape, blobs, batch, lr, x, labels, steps, mode="exact", keep_grads=False,
               acc_noise=None, optimizers=None):
    """Train K models separately on the shared batch: model k sees rows [0, batch[k]) of `x`
    and `labels` at every step (the same batch each step).  Returns a dict with
      loss  [steps, K]   pre-update losses,
      pred  list over steps of list over models of int32 [b_k],
      logits list over steps of list over models of float64 [b_k, C_k] (what `pred` is the argmax of),
      blobs list of K flat float64 weight vectors after the last step,
      grads (when keep_grads) list over steps of list over models of flat float64 gradients,
      nets  the K trained Model objects (optimiser state included).
    `optimizers`, if given, is a list of K optimiser dicts (see Model)."""
    K = len(models)
    nets = [Model(models[k], in_shape, blobs[k], mode, acc_noise, opt=(optimizers[k] if optimizers else None))
            for k in range(K)]
    loss = np.zeros((steps, K))
    preds, grads, logits = [], [], []
    for t in range(steps):
        preds.append([])
        grads.append([])
        logits.append([])
        for k, net in enumerate(nets):
            b = int(batch[k])
            l, p, g = net.sgd_step(x[:b], labels[:b], float(lr[k]))
            loss[t, k] = l
            preds[-1].append(p)
            logits[-1].append(net.last_logits)
            if keep_grads:
                grads[-1].append(Model.flatten_grads(g))
    out = {"loss": loss, "pred": preds, "logits": logits, "blobs": [n.blob() for n in nets], "nets": nets}
    if keep_grads:
        out["grads"] = grads
    return out
