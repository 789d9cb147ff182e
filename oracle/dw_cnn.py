"""Plain CPU oracle for the convolutional model: loss, gradient and Hessian-vector product.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it, and it shares no code with the HIP kernels.

The paper trains "a simple 2-layer convolutional neural network from PyTorch" (Section VI).  Reading:
the network of PyTorch's MNIST example without its dropout layers (which would make the Hessian-vector
product depend on a second random stream the paper does not mention):

    x [B,H,W,C0] -> conv 3x3 (C1) -> ReLU -> conv 3x3 (C2) -> ReLU -> max-pool 2x2 -> flatten
      -> linear (d1) -> ReLU -> ... -> linear (classes) -> softmax cross-entropy (mean over B)

Convolutions have stride 1 and no padding; the pooled map must have even height and width.
Activations are kept channels-last; the flattened vector runs over (row, column, channel).

Parameter layout (the index space of z): for each convolution W [C_out][C_in][3][3] then b [C_out];
then for each linear layer W [d_l][d_{l-1}] then b_l, as in the MLP oracle.

The Hessian-vector product is the directional derivative of the back-propagated gradient along z
(Pearlmutter's R-operator), every step of forward and backward differentiated by hand:
convolution and linear layers by the product rule, ReLU and max-pool by freezing their selections
(their second derivative is zero almost everywhere; Section IV-B's Hutchinson estimate uses H z).

AdaHessian's spatial averaging (Section IV-B, last paragraph) is, for a convolution kernel, the mean
of D = z * Hz over the 3x3 window of each (output, input) channel pair; linear layers and biases are
not averaged.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

F64 = np.float64


@dataclass(frozen=True)
class CnnSpec:
    img: Tuple[int, int, int]            # H, W, C0
    conv: Tuple[int, ...]                # output channels of the 3x3 convolutions
    fc: Tuple[int, ...]                  # widths of the linear layers after the flatten; the last is the class count

    def conv_shapes(self) -> List[Tuple[int, int, int]]:
        """(H, W, C) of the input and of every convolution's output."""
        h, w, c = self.img
        out = [(h, w, c)]
        for co in self.conv:
            h, w, c = h - 2, w - 2, co
            out.append((h, w, c))
        return out

    @property
    def flat(self) -> int:
        h, w, c = self.conv_shapes()[-1]
        assert h % 2 == 0 and w % 2 == 0
        return (h // 2) * (w // 2) * c

    def offsets(self):
        """[(w_off, b_off, w_shape)] for all layers in order (convolutions, then linear) and the total count."""
        out, pos = [], 0
        shapes = self.conv_shapes()
        for j, co in enumerate(self.conv):
            ci = shapes[j][2]
            out.append((pos, pos + co * ci * 9, (co, ci, 3, 3)))
            pos += co * ci * 9 + co
        d_in = self.flat
        for d in self.fc:
            out.append((pos, pos + d * d_in, (d, d_in)))
            pos += d * d_in + d
            d_in = d
        return out, pos


def unpack(theta: np.ndarray, spec: CnnSpec):
    offs, total = spec.offsets()
    assert theta.shape == (total,)
    return [(theta[w:b].reshape(shape), theta[b:b + shape[0]]) for (w, b, shape) in offs]


# ---- the layers, each with the adjoint maps its backward pass needs ---------------------------------------

def conv3x3(a: np.ndarray, W: np.ndarray) -> np.ndarray:
    """s[b,y,x,co] = sum_{ci,dy,dx} a[b,y+dy,x+dx,ci] W[co,ci,dy,dx]  (no bias)."""
    B, H, Wd, _ = a.shape
    s = np.zeros((B, H - 2, Wd - 2, W.shape[0]), dtype=F64)
    for dy in range(3):
        for dx in range(3):
            s += np.einsum("byxi,oi->byxo", a[:, dy:dy + H - 2, dx:dx + Wd - 2, :], W[:, :, dy, dx])
    return s


def conv3x3_input_grad(d: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Adjoint of conv3x3 in its input: da[b,y+dy,x+dx,ci] += sum_co d[b,y,x,co] W[co,ci,dy,dx]."""
    B, Ho, Wo, _ = d.shape
    da = np.zeros((B, Ho + 2, Wo + 2, W.shape[1]), dtype=F64)
    for dy in range(3):
        for dx in range(3):
            da[:, dy:dy + Ho, dx:dx + Wo, :] += np.einsum("byxo,oi->byxi", d, W[:, :, dy, dx])
    return da


def conv3x3_weight_grad(d: np.ndarray, a: np.ndarray) -> np.ndarray:
    """Adjoint of conv3x3 in its kernel: gW[co,ci,dy,dx] = sum_{b,y,x} d[b,y,x,co] a[b,y+dy,x+dx,ci]."""
    B, Ho, Wo, Co = d.shape
    g = np.zeros((Co, a.shape[3], 3, 3), dtype=F64)
    for dy in range(3):
        for dx in range(3):
            g[:, :, dy, dx] = np.einsum("byxo,byxi->oi", d, a[:, dy:dy + Ho, dx:dx + Wo, :])
    return g


def maxpool2(a: np.ndarray):
    """2x2 max-pool; returns the pooled map and, per output, which of the four inputs was taken
    (0..3 in the order (0,0), (0,1), (1,0), (1,1); the first one on ties)."""
    B, H, W, C = a.shape
    win = a.reshape(B, H // 2, 2, W // 2, 2, C).transpose(0, 1, 3, 5, 2, 4).reshape(B, H // 2, W // 2, C, 4)
    idx = np.argmax(win, axis=-1)                    # first maximum
    return np.take_along_axis(win, idx[..., None], axis=-1)[..., 0], idx


def pool_select(a: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """The pooled map of `a` taking the inputs recorded in idx (used for the directional derivative)."""
    B, H, W, C = a.shape
    win = a.reshape(B, H // 2, 2, W // 2, 2, C).transpose(0, 1, 3, 5, 2, 4).reshape(B, H // 2, W // 2, C, 4)
    return np.take_along_axis(win, idx[..., None], axis=-1)[..., 0]


def unpool2(d: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Adjoint of pool_select: route d back to the recorded inputs, zeros elsewhere."""
    B, Hp, Wp, C = d.shape
    win = np.zeros((B, Hp, Wp, C, 4), dtype=F64)
    np.put_along_axis(win, idx[..., None], d[..., None], axis=-1)
    return win.reshape(B, Hp, Wp, C, 2, 2).transpose(0, 1, 4, 2, 5, 3).reshape(B, Hp * 2, Wp * 2, C)


def softmax_rows(s):
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


# ---- loss, gradient, Hessian-vector product ----------------------------------------------------------------

def loss_only(theta, x, y, spec: CnnSpec) -> float:
    layers = unpack(np.asarray(theta, dtype=F64), spec)
    a = np.asarray(x, dtype=F64)
    nc = len(spec.conv)
    for (W, b) in layers[:nc]:
        a = np.maximum(conv3x3(a, W) + b, 0.0)
    a, _ = maxpool2(a)
    a = a.reshape(a.shape[0], -1)
    for l, (W, b) in enumerate(layers[nc:]):
        s = a @ W.T + b
        a = np.maximum(s, 0.0) if l < len(spec.fc) - 1 else s
    p = softmax_rows(a)
    return float(-np.mean(np.log(p[np.arange(len(y)), y])))


def grad_and_hvp(theta, x, y, spec: CnnSpec, z=None):
    """Mean minibatch loss, its gradient g and (when z is given) the Hessian-vector product H z,
    all in the parameter layout of the module header.  Also returns the smallest |pre-activation|
    met at a ReLU and the smallest gap between the two largest entries of a pooling window (how far
    the point is from a kink)."""
    theta = np.asarray(theta, dtype=F64)
    x = np.asarray(x, dtype=F64)
    B = x.shape[0]
    layers = unpack(theta, spec)
    dirs = unpack(np.asarray(z, dtype=F64), spec) if z is not None else [(np.zeros_like(W), np.zeros_like(b))
                                                                           for (W, b) in layers]
    nc, nf = len(spec.conv), len(spec.fc)
    margin = np.inf

    # forward and its derivative along z (R-forward)
    acts, racts, pre = [x], [np.zeros_like(x)], []
    for j in range(nc):
        (W, b), (V, c) = layers[j], dirs[j]
        s = conv3x3(acts[-1], W) + b
        rs = conv3x3(racts[-1], W) + conv3x3(acts[-1], V) + c
        on = s > 0.0
        margin = min(margin, float(np.abs(s).min()))
        pre.append(on)
        acts.append(np.where(on, s, 0.0)); racts.append(np.where(on, rs, 0.0))
    pooled, idx = maxpool2(acts[-1])
    srt = np.sort(acts[-1].reshape(B, pooled.shape[1], 2, pooled.shape[2], 2, -1).transpose(0, 1, 3, 5, 2, 4)
                  .reshape(B, pooled.shape[1], pooled.shape[2], -1, 4), axis=-1)
    live = srt[..., 3] > 0.0                          # windows whose maximum is not the clipped zero
    if live.any():
        margin = min(margin, float((srt[..., 3] - srt[..., 2])[live].min()))
    rpooled = pool_select(racts[-1], idx)
    f, rf = [pooled.reshape(B, -1)], [rpooled.reshape(B, -1)]
    fpre = []
    for l in range(nf):
        (W, b), (V, c) = layers[nc + l], dirs[nc + l]
        s = f[-1] @ W.T + b
        rs = rf[-1] @ W.T + f[-1] @ V.T + c
        if l < nf - 1:
            on = s > 0.0
            margin = min(margin, float(np.abs(s).min()))
            fpre.append(on)
            f.append(np.where(on, s, 0.0)); rf.append(np.where(on, rs, 0.0))
        else:
            logits, rlogits = s, rs
    p = softmax_rows(logits)
    loss = float(-np.mean(np.log(p[np.arange(B), y])))

    # backward and its derivative along z (R-backward)
    onehot = np.zeros_like(p); onehot[np.arange(B), y] = 1.0
    d = (p - onehot) / B
    rd = p * (rlogits - np.sum(p * rlogits, axis=1, keepdims=True)) / B
    g, hz = np.zeros_like(theta), np.zeros_like(theta)
    offs, _ = spec.offsets()
    for l in range(nf - 1, -1, -1):
        (W, b), (V, c) = layers[nc + l], dirs[nc + l]
        w_off, b_off, shape = offs[nc + l]
        g[w_off:b_off] = (d.T @ f[l]).reshape(-1)
        hz[w_off:b_off] = (rd.T @ f[l] + d.T @ rf[l]).reshape(-1)
        g[b_off:b_off + shape[0]] = d.sum(axis=0)
        hz[b_off:b_off + shape[0]] = rd.sum(axis=0)
        d_in, rd_in = d @ W, rd @ W + d @ V
        if l > 0:
            d, rd = np.where(fpre[l - 1], d_in, 0.0), np.where(fpre[l - 1], rd_in, 0.0)
        else:
            d, rd = d_in, rd_in
    # through the flatten and the pooling, then the ReLU of the last convolution
    d = unpool2(d.reshape(pooled.shape), idx)
    rd = unpool2(rd.reshape(pooled.shape), idx)
    for j in range(nc - 1, -1, -1):
        (W, b), (V, c) = layers[j], dirs[j]
        w_off, b_off, shape = offs[j]
        d, rd = np.where(pre[j], d, 0.0), np.where(pre[j], rd, 0.0)
        g[w_off:b_off] = conv3x3_weight_grad(d, acts[j]).reshape(-1)
        hz[w_off:b_off] = (conv3x3_weight_grad(rd, acts[j]) + conv3x3_weight_grad(d, racts[j])).reshape(-1)
        g[b_off:b_off + shape[0]] = d.sum(axis=(0, 1, 2))
        hz[b_off:b_off + shape[0]] = rd.sum(axis=(0, 1, 2))
        if j > 0:
            d, rd = conv3x3_input_grad(d, W), conv3x3_input_grad(rd, W) + conv3x3_input_grad(d, V)
    return loss, g, (hz if z is not None else None), margin


def spatial_average(D: np.ndarray, spec: CnnSpec) -> np.ndarray:
    """Mean of D over the 3x3 window of every (output, input) channel pair of the convolutions;
    linear layers and all biases are left as they are."""
    out = np.asarray(D, dtype=F64).copy()
    offs, _ = spec.offsets()
    for j in range(len(spec.conv)):
        w_off, b_off, _ = offs[j]
        blk = out[w_off:b_off].reshape(-1, 9).mean(axis=1, keepdims=True)
        out[w_off:b_off] = np.broadcast_to(blk, (blk.shape[0], 9)).reshape(-1)
    return out
