"""CPU oracle for a slide training step with a convolutional (ResNet) tile encoder.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this module; the product
path never does, and it shares no code with the HIP path.

What it computes (paper, Method: any tile encoder followed by the aggregator; Results: the
gradient-equivalence, EGFR and whole-slide breast experiments use ResNet50 / ResNet18 encoders
under the gated-attention aggregator): every tile goes through a residual convolutional network,
the global average of its last feature map is the tile's feature row, the feature matrix goes
through the aggregator and criterion of slide_oracle.pool_fwd, and the loss is differentiated with
respect to every parameter.  The method is exact, so the oracle is the definition written out in
float64: forward of the composed function, then reverse-mode derivatives step by step.  A
convolution is the sum over its taps of a channel contraction (library tensordot) of a shifted,
strided view of the zero-padded input; nothing is blocked, fused or reordered.

Network (the paper names the architectures only; taken: the standard residual networks of He et
al. as commonly implemented): 7x7 stride-2 convolution with 64 channels, batch normalisation, ReLU,
3x3 stride-2 max pooling with padding 1; four stages of residual blocks (basic: 3x3, 3x3;
bottleneck: 1x1, 3x3 carrying the stride, 1x1 with four-fold expansion), a 1x1 convolution +
batch normalisation on the shortcut wherever stride or width changes; global average pooling; no
classification layer (the aggregator takes its place).  Convolutions carry no bias.

Batch normalisation uses the statistics of the batch it sees, biased variance, over all tiles of
the call and all positions (Results, gradient equivalence: the normalisation layers were
synchronised across devices so that the statistics are those of the whole slide; on one device
that is the plain batch statistic over every tile of the slide).

Storage precision.  The paper trains these encoders with 16-bit mixed precision (Method, the
tiles-per-device figures with automatic mixed precision), and a ReLU or a max pooling turns a
floating-point value into a decision (which inputs pass a gradient).  For a comparison with a path
that stores its activations in 16 bits both sides must take those decisions on the same numbers, so
every function here takes `store`: a function applied to each activation tensor at the point where a
16-bit path writes it to memory (convolution outputs; outputs of normalisation + ReLU; block outputs
behind the residual sum and ReLU).  The default is the identity (plain float64: the definition);
the parity tests of the bfloat16 path pass round-to-nearest-even to bfloat16.  Arithmetic between
two such points stays float64, and nothing is rounded in the backward.

Parity pins: tests/test_oracle_resnet.py (finite differences of the scalar loss, an independent
autograd graph of library routines, brute-force loops, 1x1 convolution = matrix product,
normalisation invariants, pooling routing).  Nothing is "parity unpinned".

Parameters are a dict name -> ndarray, names and shapes as gen.resnet_param_shapes.
"""
from __future__ import annotations

import numpy as np

from .slide_oracle import pool_fwd, pool_bwd


# ----------------------------------------------------------------------------
# elementary pieces (x is [n, C, H, W])
# ----------------------------------------------------------------------------

def conv2d_fwd(x, W, stride, pad):
    """out[n,o,y,x] = sum_{c,kh,kw} W[o,c,kh,kw] * xpad[n,c,y*stride+kh,x*stride+kw]."""
    n, C, H, Wd = x.shape
    O, _, KH, KW = W.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (Wd + 2 * pad - KW) // stride + 1
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    out = np.zeros((n, O, OH, OW), dtype=x.dtype)
    for kh in range(KH):
        for kw in range(KW):
            v = xp[:, :, kh:kh + stride * (OH - 1) + 1:stride, kw:kw + stride * (OW - 1) + 1:stride]
            out += np.tensordot(v, W[:, :, kh, kw], axes=([1], [1])).transpose(0, 3, 1, 2)
    return out


def conv2d_bwd(dout, x, W, stride, pad):
    """Gradients of conv2d_fwd with respect to its input and its weights."""
    n, C, H, Wd = x.shape
    O, _, KH, KW = W.shape
    OH, OW = dout.shape[2], dout.shape[3]
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    dxp = np.zeros_like(xp)
    dW = np.zeros_like(W)
    for kh in range(KH):
        for kw in range(KW):
            ys = slice(kh, kh + stride * (OH - 1) + 1, stride)
            xs = slice(kw, kw + stride * (OW - 1) + 1, stride)
            v = xp[:, :, ys, xs]
            dW[:, :, kh, kw] = np.tensordot(dout, v, axes=([0, 2, 3], [0, 2, 3]))
            dxp[:, :, ys, xs] += np.tensordot(dout, W[:, :, kh, kw], axes=([1], [0])).transpose(0, 3, 1, 2)
    dx = dxp[:, :, pad:pad + H, pad:pad + Wd]
    return dx, dW


def bn_fwd(x, g, b, eps):
    """Batch normalisation with the statistics of this batch (biased variance over n, H, W)."""
    mu = x.mean(axis=(0, 2, 3), keepdims=True)
    var = ((x - mu) ** 2).mean(axis=(0, 2, 3), keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    return xh * g[None, :, None, None] + b[None, :, None, None], (xh, rstd)


def bn_bwd(dy, g, cache):
    xh, rstd = cache
    dxh = dy * g[None, :, None, None]
    dx = rstd * (dxh - dxh.mean(axis=(0, 2, 3), keepdims=True)
                 - xh * (dxh * xh).mean(axis=(0, 2, 3), keepdims=True))
    return dx, (dy * xh).sum(axis=(0, 2, 3)), dy.sum(axis=(0, 2, 3))


def maxpool_fwd(x):
    """3x3 window, stride 2, padding 1 (padding never wins).  Of equal maxima the first in
    (kh, kw) scan order takes the gradient."""
    n, C, H, W = x.shape
    OH, OW = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)), constant_values=-np.inf)
    taps = np.stack([xp[:, :, kh:kh + 2 * (OH - 1) + 1:2, kw:kw + 2 * (OW - 1) + 1:2]
                     for kh in range(3) for kw in range(3)], axis=0)
    arg = taps.argmax(axis=0)
    return np.take_along_axis(taps, arg[None], axis=0)[0], (arg, x.shape)


def maxpool_bwd(dout, cache):
    arg, shape = cache
    n, C, H, W = shape
    OH, OW = dout.shape[2], dout.shape[3]
    dxp = np.zeros((n, C, H + 2, W + 2), dtype=dout.dtype)
    for t in range(9):
        kh, kw = divmod(t, 3)
        dxp[:, :, kh:kh + 2 * (OH - 1) + 1:2, kw:kw + 2 * (OW - 1) + 1:2] += np.where(arg == t, dout, 0.0)
    return dxp[:, :, 1:1 + H, 1:1 + W]


# ----------------------------------------------------------------------------
# network
# ----------------------------------------------------------------------------

def _blocks(cfg):
    out = []
    cin = cfg.width
    exp = 1 if cfg.block == "basic" else 4
    for s, depth in enumerate(cfg.depths):
        mid = cfg.width * (2 ** s)
        cout = mid * exp
        for b in range(depth):
            stride = 2 if (b == 0 and s > 0) else 1
            out.append((f"s{s}.b{b}", stride, stride != 1 or cin != cout))
            cin = cout
    return out


def _identity(a):
    return a


def _conv_bn(P, x, conv, bn, stride, pad, eps, store):
    c = store(conv2d_fwd(x, P[conv + ".W"], stride, pad))
    y, bc = bn_fwd(c, P[bn + ".g"], P[bn + ".b"], eps)
    return y, (x, conv, bn, stride, pad, bc)


def _conv_bn_bwd(P, g, dy, cache):
    x, conv, bn, stride, pad, bc = cache
    dc, g[bn + ".g"], g[bn + ".b"] = bn_bwd(dy, P[bn + ".g"], bc)
    dx, g[conv + ".W"] = conv2d_bwd(dc, x, P[conv + ".W"], stride, pad)
    return dx


def encoder_fwd(prm, X, cfg, dtype=np.float64, store=_identity):
    """Tile features H [n, dim] and the cache for encoder_bwd.  X: [n,3,S,S] normalised pixels."""
    P = {k: np.asarray(v, dtype=dtype) for k, v in prm.items() if not k.startswith(("mil.", "head."))}
    eps = cfg.bn_eps
    x = np.asarray(X, dtype=dtype)
    y, c0 = _conv_bn(P, x, "stem.conv", "stem.bn", 2, 3, eps, store)
    r0 = store(np.maximum(y, 0.0))
    x, mp = maxpool_fwd(r0)
    caches = []
    for name, stride, down in _blocks(cfg):
        p = name + "."
        x0 = x
        if cfg.block == "basic":
            y1, k1 = _conv_bn(P, x0, p + "conv1", p + "bn1", stride, 1, eps, store)
            r1 = store(np.maximum(y1, 0.0))
            y2, k2 = _conv_bn(P, r1, p + "conv2", p + "bn2", 1, 1, eps, store)
            body, ks, rs = y2, [k1, k2], [r1]
        else:
            y1, k1 = _conv_bn(P, x0, p + "conv1", p + "bn1", 1, 0, eps, store)
            r1 = store(np.maximum(y1, 0.0))
            y2, k2 = _conv_bn(P, r1, p + "conv2", p + "bn2", stride, 1, eps, store)
            r2 = store(np.maximum(y2, 0.0))
            y3, k3 = _conv_bn(P, r2, p + "conv3", p + "bn3", 1, 0, eps, store)
            body, ks, rs = y3, [k1, k2, k3], [r1, r2]
        if down:
            sc, kd = _conv_bn(P, x0, p + "down.conv", p + "down.bn", stride, 0, eps, store)
        else:
            sc, kd = x0, None
        x = store(np.maximum(body + sc, 0.0))
        caches.append((ks, rs, kd, x))
    H = x.mean(axis=(2, 3))
    return H, {"P": P, "stem": (c0, r0, mp), "blocks": caches, "last_shape": x.shape}


def encoder_bwd(cache, G):
    """Encoder parameter gradients for feature-gradient rows G [n, dim] (paper, Method: the
    pseudo-loss sum(G * H) back-propagated through the encoder; no rank factor on one device)."""
    P = cache["P"]
    g = {}
    n, C, Hh, Ww = cache["last_shape"]
    dx = np.broadcast_to(np.asarray(G, dtype=np.float64)[:, :, None, None] / (Hh * Ww), (n, C, Hh, Ww)).copy()
    for ks, rs, kd, out in reversed(cache["blocks"]):
        dz = np.where(out > 0.0, dx, 0.0)                 # ReLU behind the sum
        d = _conv_bn_bwd(P, g, dz, ks[-1])
        for k, r in zip(reversed(ks[:-1]), reversed(rs)):
            d = _conv_bn_bwd(P, g, np.where(r > 0.0, d, 0.0), k)
        dx = d + (_conv_bn_bwd(P, g, dz, kd) if kd is not None else dz)
    c0, r0, mp = cache["stem"]
    d = maxpool_bwd(dx, mp)
    _conv_bn_bwd(P, g, np.where(r0 > 0.0, d, 0.0), c0)
    return g


def slide_loss(prm, X, label, cfg, dtype=np.float64, store=_identity):
    Hf, _ = encoder_fwd(prm, X, cfg, dtype, store)
    return pool_fwd(prm, Hf, label, cfg, dtype)[0]


def slide_step(prm, X, label, cfg, dtype=np.float64, store=_identity):
    """One forward + backward step over all tiles of a slide: dict(loss, logits, alpha, H, G, grads)."""
    Hf, cache = encoder_fwd(prm, X, cfg, dtype, store)
    loss, y, alpha, z, pc = pool_fwd(prm, Hf, label, cfg, dtype)
    G, grads = pool_bwd(pc)
    grads.update(encoder_bwd(cache, G))
    return {"loss": loss, "logits": y, "alpha": alpha, "z": z, "H": Hf, "G": G, "grads": grads}
