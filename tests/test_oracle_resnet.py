"""Pins for the CPU oracle of the convolutional (ResNet) tile encoder: things the mathematics and
library routines fix, none of which re-use the oracle's own formulas.

* finite differences of the WHOLE scalar slide loss (pins every gradient, including the seam
  aggregator backward -> feature gradients -> encoder backward);
* an independent autograd graph of library routines (torch float64 conv2d / batch_norm in training
  mode / max_pool2d / adaptive_avg_pool2d), basic and bottleneck blocks, with and without a
  projection on the shortcut;
* brute-force scalar loops for the convolution and the max pooling on tiny inputs;
* closed forms and invariants: 1x1 convolution = matrix product, a centred one-hot kernel = identity, batch
  normalisation output moments, its input gradient is orthogonal to 1 and to the normalised input,
  invariance of a conv+BN pair under rescaling of the convolution weights, max-pool gradient routing
  and tie rule, tile permutation.
"""
from dataclasses import replace

import numpy as np
import pytest

import gen
from gen import resnet_inputs as rgen
from oracle import resnet_oracle as ro


def _case(name, n=None, n_classes=None):
    cfg, n0 = rgen.RESNET_CONFIGS[name]
    if n_classes is not None:
        cfg = replace(cfg, n_classes=n_classes)
    ds, ws, ls = rgen.RESNET_SEEDS[name]
    n = n0 if n is None else n
    prm = rgen.make_resnet_params(cfg, ws)
    X = gen.make_pixels(cfg, n, ds, kind="blur")
    rng = np.random.Generator(np.random.PCG64(ls))
    label = int(rng.random() < 0.5) if cfg.n_classes == 1 else int(rng.integers(0, cfg.n_classes))
    return cfg, {k: v.astype(np.float64) for k, v in prm.items()}, X.astype(np.float64), label


# ---------------------------------------------------------------- finite differences

def _fd(f, arr, i, h):
    old = arr[i]
    vals = []
    for k in (1, -1, 2, -2):
        arr[i] = old + k * h
        vals.append(f())
    arr[i] = old
    return (8 * (vals[0] - vals[1]) - (vals[2] - vals[3])) / (12 * h)


@pytest.mark.parametrize("name,ncls", [("rn_probe", 1), ("rn_probe", 3)])
def test_fd_whole_loss(name, ncls):
    cfg, prm, X, label = _case(name, n_classes=ncls)
    res = ro.slide_step(prm, X, label, cfg)
    f = lambda: ro.slide_loss(prm, X, label, cfg)
    rng = np.random.default_rng(5)
    worst = 0.0
    for pname, g in res["grads"].items():
        flat = prm[pname].reshape(-1)
        for i in rng.choice(flat.size, size=min(3, flat.size), replace=False):
            fd = _fd(f, flat, i, 1e-4 * max(1.0, abs(flat[i])))
            an = g.reshape(-1)[i]
            err = abs(fd - an) / max(abs(an), abs(fd), 1e-7)
            # ReLU and max pooling are piecewise linear: a coordinate whose step crosses a kink is skipped by the
            # magnitude test only if both values are tiny; otherwise the quotient must match
            assert err < 2e-5, (pname, int(i), fd, an)
            worst = max(worst, err)
    assert worst < 2e-5


# ---------------------------------------------------------------- independent autograd graph

def _torch_step(cfg, prm, X, label):
    import torch
    import torch.nn.functional as F
    torch.set_num_threads(4)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in prm.items()}
    eps = cfg.bn_eps

    def cb(x, conv, bn, stride, pad):
        y = F.conv2d(x, P[conv + ".W"], None, stride=stride, padding=pad)
        return F.batch_norm(y, None, None, P[bn + ".g"], P[bn + ".b"], training=True, momentum=0.0, eps=eps)

    x = torch.tensor(X, dtype=torch.float64)
    x = F.max_pool2d(F.relu(cb(x, "stem.conv", "stem.bn", 2, 3)), 3, 2, 1)
    for blk in rgen.resnet_blocks(cfg):
        p, s = blk["name"] + ".", blk["stride"]
        if cfg.block == "basic":
            y = cb(F.relu(cb(x, p + "conv1", p + "bn1", s, 1)), p + "conv2", p + "bn2", 1, 1)
        else:
            y = F.relu(cb(x, p + "conv1", p + "bn1", 1, 0))
            y = F.relu(cb(y, p + "conv2", p + "bn2", s, 1))
            y = cb(y, p + "conv3", p + "bn3", 1, 0)
        sc = cb(x, p + "down.conv", p + "down.bn", s, 0) if blk["down"] else x
        x = F.relu(y + sc)
    H = F.adaptive_avg_pool2d(x, 1).flatten(1)
    H.retain_grad()
    t = torch.tanh(F.linear(H, P["mil.V.W"], P["mil.V.b"]))
    sg = torch.sigmoid(F.linear(H, P["mil.U.W"], P["mil.U.b"]))
    alpha = torch.softmax((t * sg) @ P["mil.w"], dim=0)
    y = F.linear(alpha @ H, P["head.W"], P["head.b"])
    if cfg.n_classes == 1:
        loss = F.binary_cross_entropy_with_logits(y, torch.tensor([float(label)], dtype=torch.float64))
    else:
        loss = F.cross_entropy(y[None], torch.tensor([label]))
    loss.backward()
    return float(loss.detach()), H.detach().numpy(), H.grad.numpy(), {k: v.grad.numpy() for k, v in P.items()}


@pytest.mark.parametrize("name,n,ncls", [("rn_probe", 3, 1), ("rn_tiny", 3, 3), ("rn_tiny_bneck", 3, 1)])
def test_against_library_autograd(name, n, ncls):
    cfg, prm, X, label = _case(name, n=n, n_classes=ncls)
    if name != "rn_probe":
        cfg = replace(cfg, tile=32)
        X = X[:, :, :32, :32]
    res = ro.slide_step(prm, X, label, cfg)
    loss, H, G, grads = _torch_step(cfg, prm, X, label)
    assert abs(res["loss"] - loss) < 1e-12 * max(1.0, abs(loss))
    np.testing.assert_allclose(res["H"], H, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(res["G"], G, rtol=1e-8, atol=1e-13)
    assert set(res["grads"]) == set(grads)
    for k, v in grads.items():
        scale = np.abs(v).max() + 1e-300
        assert np.abs(res["grads"][k] - v).max() < 1e-9 * scale, k


def test_resnet18_and_50_layouts_run_through_library_graph():
    """The full-depth layouts (8 and 16 blocks, every stride / projection combination) at a 32 px tile."""
    for name in ("rn18_small", "rn50_small"):
        cfg, prm, X, label = _case(name, n=4)
        cfg = replace(cfg, tile=32, width=8)
        ws = rgen.RESNET_SEEDS[name][1]
        prm = {k: v.astype(np.float64) for k, v in rgen.make_resnet_params(cfg, ws).items()}
        X = X[:, :, :32, :32]
        res = ro.slide_step(prm, X, label, cfg)
        loss, H, G, grads = _torch_step(cfg, prm, X, label)
        # the last stage is one position per tile here, so its normalisations see four samples per channel: the two
        # float64 computations differ by rounding amplified through 1 / sqrt(var + eps)
        assert abs(res["loss"] - loss) < 1e-10
        for k, v in grads.items():
            assert np.abs(res["grads"][k] - v).max() < 1e-7 * (np.abs(v).max() + 1e-300), (name, k)


# ---------------------------------------------------------------- brute force

def test_convolution_against_scalar_loops():
    rng = np.random.default_rng(0)
    for (C, O, K, s, p, H, W) in [(2, 3, 3, 1, 1, 5, 4), (3, 2, 3, 2, 1, 6, 7), (2, 2, 1, 2, 0, 5, 5), (3, 2, 7, 2, 3, 9, 8)]:
        x = rng.standard_normal((2, C, H, W))
        Wt = rng.standard_normal((O, C, K, K))
        OH, OW = (H + 2 * p - K) // s + 1, (W + 2 * p - K) // s + 1
        ref = np.zeros((2, O, OH, OW))
        for n in range(2):
            for o in range(O):
                for y in range(OH):
                    for xx in range(OW):
                        acc = 0.0
                        for c in range(C):
                            for kh in range(K):
                                for kw in range(K):
                                    iy, ix = y * s + kh - p, xx * s + kw - p
                                    if 0 <= iy < H and 0 <= ix < W:
                                        acc += Wt[o, c, kh, kw] * x[n, c, iy, ix]
                        ref[n, o, y, xx] = acc
        out = ro.conv2d_fwd(x, Wt, s, p)
        np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
        # the backward is the transpose of the forward in both arguments: <dout, conv(x, W)> is bilinear
        dout = rng.standard_normal(out.shape)
        dx, dW = ro.conv2d_bwd(dout, x, Wt, s, p)
        ex = rng.standard_normal(x.shape)
        eW = rng.standard_normal(Wt.shape)
        assert abs((dout * ro.conv2d_fwd(ex, Wt, s, p)).sum() - (dx * ex).sum()) < 1e-10
        assert abs((dout * ro.conv2d_fwd(x, eW, s, p)).sum() - (dW * eW).sum()) < 1e-10


def test_maxpool_against_scalar_loops_and_tie_rule():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 7, 6))
    x[0, 0, :4, :4] = 1.5          # a plateau: equal maxima inside windows
    out, cache = ro.maxpool_fwd(x)
    dout = rng.standard_normal(out.shape)
    dx = ro.maxpool_bwd(dout, cache)
    ref = np.zeros_like(out)
    dref = np.zeros_like(x)
    for n in range(2):
        for c in range(3):
            for y in range(out.shape[2]):
                for xx in range(out.shape[3]):
                    best, at = -np.inf, None
                    for kh in range(3):
                        for kw in range(3):
                            iy, ix = 2 * y + kh - 1, 2 * xx + kw - 1
                            if 0 <= iy < 7 and 0 <= ix < 6 and x[n, c, iy, ix] > best:   # strict: first maximum wins
                                best, at = x[n, c, iy, ix], (iy, ix)
                    ref[n, c, y, xx] = best
                    dref[n, c, at[0], at[1]] += dout[n, c, y, xx]
    np.testing.assert_array_equal(out, ref)
    np.testing.assert_allclose(dx, dref, rtol=0, atol=1e-15)
    assert abs(dx.sum() - dout.sum()) < 1e-12      # every output routes its gradient to exactly one input


# ---------------------------------------------------------------- closed forms and invariants

def test_pointwise_convolution_is_a_matrix_product_and_delta_kernel_is_identity():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 5, 4, 3))
    W = rng.standard_normal((6, 5, 1, 1))
    out = ro.conv2d_fwd(x, W, 1, 0)
    np.testing.assert_allclose(out, np.einsum("oc,nchw->nohw", W[:, :, 0, 0], x), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ro.conv2d_fwd(x, W, 2, 0), out[:, :, ::2, ::2], rtol=1e-13, atol=1e-13)
    D = np.zeros((5, 5, 3, 3))
    D[np.arange(5), np.arange(5), 1, 1] = 1.0
    np.testing.assert_array_equal(ro.conv2d_fwd(x, D, 1, 1), x)
    S = np.zeros((5, 5, 3, 3))
    S[np.arange(5), np.arange(5), 0, 2] = 1.0      # tap (kh=0, kw=2): out[y, x] = in[y - 1, x + 1]
    sh = ro.conv2d_fwd(x, S, 1, 1)
    np.testing.assert_array_equal(sh[:, :, 1:, :-1], x[:, :, :-1, 1:])
    assert not sh[:, :, 0, :].any() and not sh[:, :, :, -1].any()


def test_batchnorm_moments_and_gradient_orthogonality():
    rng = np.random.default_rng(3)
    x = 3.0 + 2.0 * rng.standard_normal((4, 3, 5, 6))
    g = rng.standard_normal(3)
    b = rng.standard_normal(3)
    y, cache = ro.bn_fwd(x, g, b, 1e-5)
    xh = cache[0]
    assert np.abs(xh.mean(axis=(0, 2, 3))).max() < 1e-13
    var = x.var(axis=(0, 2, 3))
    np.testing.assert_allclose(xh.var(axis=(0, 2, 3)), var / (var + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(y, xh * g[None, :, None, None] + b[None, :, None, None], rtol=1e-13)
    dy = rng.standard_normal(y.shape)
    dx, dg, db = ro.bn_bwd(dy, g, cache)
    # the output does not change when a constant is added to x or x is scaled about its mean: the input gradient is
    # orthogonal to both directions
    assert np.abs(dx.sum(axis=(0, 2, 3))).max() < 1e-12
    assert np.abs((dx * xh).sum(axis=(0, 2, 3))).max() < 1e-4      # exact only for eps = 0
    _, c0 = ro.bn_fwd(x, g, b, 0.0)
    dx0, _, _ = ro.bn_bwd(dy, g, c0)
    assert np.abs((dx0 * c0[0]).sum(axis=(0, 2, 3))).max() < 1e-11
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), rtol=1e-13)


def test_conv_bn_pair_ignores_weight_scale():
    cfg, prm, X, label = _case("rn_probe")
    a = ro.slide_loss(prm, X, label, replace(cfg, bn_eps=0.0))
    prm2 = dict(prm)
    prm2["s1.b0.conv1.W"] = prm["s1.b0.conv1.W"] * 3.7
    prm2["stem.conv.W"] = prm["stem.conv.W"] * 0.21
    b = ro.slide_loss(prm2, X, label, replace(cfg, bn_eps=0.0))
    assert abs(a - b) < 1e-10
    # hence the weight gradient is orthogonal to the weight itself
    g = ro.slide_step(prm, X, label, replace(cfg, bn_eps=0.0))["grads"]
    for k in ("stem.conv.W", "s1.b0.conv1.W", "s3.b0.down.conv.W"):
        assert abs((g[k] * prm[k]).sum()) < 1e-10 * np.abs(g[k]).sum(), k


def test_tile_permutation_and_shapes():
    cfg, prm, X, label = _case("rn_probe")
    r = ro.slide_step(prm, X, label, cfg)
    assert r["H"].shape == (X.shape[0], cfg.dim) and (r["H"] >= 0).all()      # features are averages of ReLU outputs
    perm = np.array([2, 0, 1])
    r2 = ro.slide_step(prm, X[perm], label, cfg)
    assert abs(r["loss"] - r2["loss"]) < 1e-12
    np.testing.assert_allclose(r2["H"], r["H"][perm], rtol=1e-11, atol=1e-13)
    for k, v in r["grads"].items():
        np.testing.assert_allclose(r2["grads"][k], v, rtol=1e-8, atol=1e-12 * (np.abs(v).max() + 1e-300))
    assert set(r["grads"]) == {n for n, _ in rgen.resnet_param_shapes(cfg)}
    for n, shp in rgen.resnet_param_shapes(cfg):
        assert r["grads"][n].shape == tuple(shp), n


def test_batch_statistics_couple_the_tiles():
    """The normalisation statistics run over every tile of the call: the features of a tile depend on the others, so
    (unlike the transformer encoder) the step over a slide is not the sum of steps over chunks of it."""
    cfg, prm, X, label = _case("rn_probe")
    H_all = ro.encoder_fwd(prm, X, cfg)[0]
    H_two = ro.encoder_fwd(prm, X[:2], cfg)[0]
    assert np.abs(H_all[:2] - H_two).max() > 1e-3


def test_storage_hook_points_and_default():
    """`store` is applied exactly where a 16-bit path writes an activation (every convolution output, every ReLU
    output), the default is the plain float64 definition, and with rounding to bfloat16 the masks of the backward are
    taken on the rounded values."""
    cfg, prm, X, label = _case("rn_probe")
    seen = []

    def spy(a):
        seen.append(a.shape)
        return a

    plain = ro.slide_step(prm, X, label, cfg)
    spied = ro.slide_step(prm, X, label, cfg, store=spy)
    assert plain["loss"] == spied["loss"]
    for k, v in plain["grads"].items():
        assert np.array_equal(v, spied["grads"][k]), k
    blocks = rgen.resnet_blocks(cfg)
    convs = 1 + sum(2 + int(b["down"]) for b in blocks)      # basic blocks
    relus = 1 + 2 * len(blocks)
    assert len(seen) == convs + relus

    def bf16(a):
        return gen.to_bf16_grid(a.astype(np.float32)).astype(np.float64)

    H, cache = ro.encoder_fwd(prm, X, cfg, store=bf16)
    for ks, rs, kd, out in cache["blocks"]:
        for t in rs + [out]:
            assert np.array_equal(t, bf16(t))
    rel = np.linalg.norm(H - plain["H"]) / np.linalg.norm(plain["H"])
    assert 1e-4 < rel < 5e-2      # 16-bit storage moves the features by a fraction of a percent, not more
