"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which re-use the oracle's own formulas.

* finite differences of the WHOLE scalar slide loss (pins every gradient and
  the pool-backward -> G -> encoder-backward seam, i.e. the pseudo-loss identity
  of the paper's Method section);
* an independent autograd graph built from library routines (torch float64
  layer_norm / gelu / softmax / linear / BCE / CE);
* a deliberately naive scalar-loop forward on a tiny case (pins patch order,
  head slicing, token layout);
* closed forms and invariants (N=1, w=0 mean pooling, permutation of tiles,
  chunk additivity = the paper's single- vs multi-device equivalence, zero
  K-bias gradient, loss at zero logits, depth-0 encoder, max-pool limit).
"""
import math
from dataclasses import replace

import numpy as np
import pytest

import gen
from oracle import slide_oracle as so


def _case(name, perturbed=True, n=None, n_classes=None, kind=None, std=0.02):
    cfg, n0 = gen.CONFIGS[name]
    if n_classes is not None:
        cfg = replace(cfg, n_classes=n_classes)
    ds, ws, ls = gen.SEEDS[name]
    n = n0 if n is None else n
    prm = gen.make_params(cfg, ws, perturbed=perturbed, std=std)
    X = gen.make_pixels(cfg, n, ds, kind=kind or ("uniform" if name in ("probe", "tiny") else "blur"))
    return cfg, prm, X.astype(np.float64), gen.make_label(cfg, ls)


# ---------------------------------------------------------------- finite differences

def _fd(f, arr, i, h):
    """4-point central difference (error O(h^4)) of scalar f() w.r.t. arr[i]."""
    old = arr[i]
    vals = []
    for k in (1, -1, 2, -2):
        arr[i] = old + k * h
        vals.append(f())
    arr[i] = old
    return (8 * (vals[0] - vals[1]) - (vals[2] - vals[3])) / (12 * h)


def _fd_check(cfg, prm, X, label, n_coord, n_pix, rng):
    prm = {k: v.astype(np.float64) for k, v in prm.items()}
    res = so.slide_step(prm, X, label, cfg)
    f = lambda: so.slide_loss(prm, X, label, cfg)
    # round-off floor of the difference quotient: ~ eps_machine * |loss| / h
    floor = 2e-11
    for name, g in res["grads"].items():
        flat = prm[name].reshape(-1)
        idx = rng.choice(flat.size, size=min(n_coord, flat.size), replace=False)
        for i in idx:
            fd = _fd(f, flat, i, 1e-4 * max(1.0, abs(flat[i])))
            an = g.reshape(-1)[i]
            scale = max(abs(an), float(np.abs(g).max()) * 1e-3)
            assert abs(fd - an) <= 2e-6 * scale + floor, (name, int(i), fd, an)
    Xf = X.reshape(-1)
    dX = res["dX"].reshape(-1)
    for i in rng.choice(Xf.size, size=n_pix, replace=False):
        fd = _fd(f, Xf, i, 1e-4)
        scale = max(abs(dX[i]), float(np.abs(dX).max()) * 1e-3)
        assert abs(fd - dX[i]) <= 2e-6 * scale + floor, ("pixel", int(i), fd, dX[i])
    # the floor must not swallow the check: typical gradients sit far above it
    big = [np.abs(g).max() for g in res["grads"].values()]
    assert np.median(big) > 1e4 * floor, np.median(big)


def test_fd_whole_loss_probe_binary():
    cfg, prm, X, label = _case("probe", std=0.3)
    _fd_check(cfg, prm, X, label, n_coord=32, n_pix=64, rng=np.random.default_rng(1))


def test_fd_whole_loss_probe_multiclass():
    cfg, prm, X, _ = _case("probe", n_classes=4, std=0.3)
    _fd_check(cfg, prm, X, 2, n_coord=32, n_pix=32, rng=np.random.default_rng(2))


def test_fd_whole_loss_tiny():
    cfg, prm, X, label = _case("tiny", std=0.1)
    _fd_check(cfg, prm, X, label, n_coord=6, n_pix=32, rng=np.random.default_rng(3))


def test_fd_vit_s_shaped_two_tiles():
    # ViT-S head/width ratios (d_h = 64, 6 heads) on 2 tiles, 2 layers, 32-px tiles
    cfg = gen.SlideConfig(32, 16, 384, 2, 6, 4, 128, 1)
    prm = gen.make_params(cfg, 77, perturbed=True, std=0.05)
    X = gen.make_pixels(cfg, 2, 78, kind="blur").astype(np.float64)
    _fd_check(cfg, prm, X, 1, n_coord=3, n_pix=16, rng=np.random.default_rng(4))


# ---------------------------------------------------------------- library autograd graph

def _torch_step(cfg, prm, X, label):
    import torch
    import torch.nn.functional as F
    tp = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in prm.items()}
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    n, D, Hh, P = X.shape[0], cfg.dim, cfg.heads, cfg.patch
    tok = F.conv2d(Xt, tp["pe.W"].reshape(D, 3, P, P), tp["pe.b"], stride=P)  # n D g g
    tok = tok.flatten(2).transpose(1, 2)
    x = torch.cat([tp["cls"].expand(n, 1, D), tok], dim=1) + tp["pos"]
    for l in range(cfg.layers):
        p = f"l{l}."
        u = F.layer_norm(x, (D,), tp[p + "ln1.g"], tp[p + "ln1.b"], cfg.ln_eps)
        qkv = F.linear(u, tp[p + "qkv.W"], tp[p + "qkv.b"])
        q, k, v = [t.reshape(n, -1, Hh, D // Hh).transpose(1, 2) for t in qkv.chunk(3, dim=-1)]
        o = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(n, -1, D)
        x = x + F.linear(o, tp[p + "proj.W"], tp[p + "proj.b"])
        u2 = F.layer_norm(x, (D,), tp[p + "ln2.g"], tp[p + "ln2.b"], cfg.ln_eps)
        x = x + F.linear(F.gelu(F.linear(u2, tp[p + "fc1.W"], tp[p + "fc1.b"])), tp[p + "fc2.W"], tp[p + "fc2.b"])
    h = F.layer_norm(x[:, 0], (D,), tp["lnf.g"], tp["lnf.b"], cfg.ln_eps)
    h.retain_grad()
    a = (torch.tanh(F.linear(h, tp["mil.V.W"], tp["mil.V.b"])) *
         torch.sigmoid(F.linear(h, tp["mil.U.W"], tp["mil.U.b"]))) @ tp["mil.w"]
    alpha = torch.softmax(a, dim=0)
    z = alpha @ h
    y = F.linear(z, tp["head.W"], tp["head.b"])
    if cfg.n_classes == 1:
        loss = F.binary_cross_entropy_with_logits(y, torch.tensor([float(label)], dtype=torch.float64))
    else:
        loss = F.cross_entropy(y[None], torch.tensor([label]))
    loss.backward()
    return loss.item(), y.detach().numpy(), alpha.detach().numpy(), h.detach().numpy(), h.grad.numpy(), \
        {k: v.grad.numpy() for k, v in tp.items()}, Xt.grad.numpy()


@pytest.mark.parametrize("name,ncls,label", [("tiny", 1, 1), ("tiny", 1, 0), ("tiny", 4, 3), ("probe", 1, 0)])
def test_against_library_autograd(name, ncls, label):
    cfg, prm, X, _ = _case(name, n_classes=ncls)
    res = so.slide_step(prm, X, label, cfg)
    loss, y, alpha, h, G, grads, dX = _torch_step(cfg, prm, X, label)
    assert abs(res["loss"] - loss) < 1e-12
    np.testing.assert_allclose(res["logits"], y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["alpha"], alpha, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(res["H"], h, rtol=0, atol=1e-11)
    np.testing.assert_allclose(res["G"], G, rtol=0, atol=1e-13)
    np.testing.assert_allclose(res["dX"], dX, rtol=0, atol=1e-13 + 1e-9 * np.abs(dX).max())
    for k, g in grads.items():
        ref = np.abs(g).max()
        assert np.abs(res["grads"][k] - g).max() <= 1e-9 * ref + 1e-15, k


def test_library_autograd_vit_s_layout():
    # 6 heads of 64: pins the q|k|v row order and the per-head column slicing at ViT-S ratios
    cfg = gen.SlideConfig(32, 16, 384, 1, 6, 4, 128, 1)
    prm = gen.make_params(cfg, 5, perturbed=True)
    X = gen.make_pixels(cfg, 3, 6).astype(np.float64)
    res = so.slide_step(prm, X, 1, cfg)
    loss, y, alpha, h, G, grads, dX = _torch_step(cfg, prm, X, 1)
    assert abs(res["loss"] - loss) < 1e-12
    for k, g in grads.items():
        assert np.abs(res["grads"][k] - g).max() <= 1e-9 * np.abs(g).max() + 1e-15, k


# ---------------------------------------------------------------- naive scalar loops

def _naive_forward(cfg, prm, X, label):
    """Scalar-loop forward; every index written out, no array arithmetic."""
    P = {k: np.asarray(v, dtype=np.float64) for k, v in prm.items()}
    n, D, Hh, Pp = X.shape[0], cfg.dim, cfg.heads, cfg.patch
    g = cfg.tile // Pp
    T = g * g + 1
    dh = D // Hh
    Fd = cfg.mlp_ratio * D

    def ln(vec, gam, bet):
        mu = sum(vec) / len(vec)
        var = sum((t - mu) ** 2 for t in vec) / len(vec)
        return [(t - mu) / math.sqrt(var + cfg.ln_eps) * gam[i] + bet[i] for i, t in enumerate(vec)]

    feats = []
    for t_ in range(n):
        x = [[0.0] * D for _ in range(T)]
        for d in range(D):
            x[0][d] = P["cls"][d] + P["pos"][0][d]
        for gy in range(g):
            for gx in range(g):
                tok = 1 + gy * g + gx
                for d in range(D):
                    acc = P["pe.b"][d] + P["pos"][tok][d]
                    for c in range(3):
                        for py in range(Pp):
                            for px in range(Pp):
                                acc += P["pe.W"][d][c * Pp * Pp + py * Pp + px] * X[t_][c][gy * Pp + py][gx * Pp + px]
                    x[tok][d] = acc
        for l in range(cfg.layers):
            p = f"l{l}."
            u = [ln(x[i], P[p + "ln1.g"], P[p + "ln1.b"]) for i in range(T)]
            qkv = [[P[p + "qkv.b"][o] + sum(P[p + "qkv.W"][o][d] * u[i][d] for d in range(D))
                    for o in range(3 * D)] for i in range(T)]
            att = [[0.0] * D for _ in range(T)]
            for hh in range(Hh):
                for i in range(T):
                    sc = [sum(qkv[i][hh * dh + e] * qkv[j][D + hh * dh + e] for e in range(dh)) / math.sqrt(dh)
                          for j in range(T)]
                    mx = max(sc)
                    ex = [math.exp(s_ - mx) for s_ in sc]
                    Z = sum(ex)
                    for e in range(dh):
                        att[i][hh * dh + e] = sum(ex[j] / Z * qkv[j][2 * D + hh * dh + e] for j in range(T))
            for i in range(T):
                for d in range(D):
                    x[i][d] += P[p + "proj.b"][d] + sum(P[p + "proj.W"][d][e] * att[i][e] for e in range(D))
            for i in range(T):
                u2 = ln(x[i], P[p + "ln2.g"], P[p + "ln2.b"])
                m = [P[p + "fc1.b"][f] + sum(P[p + "fc1.W"][f][d] * u2[d] for d in range(D)) for f in range(Fd)]
                a = [0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in m]
                for d in range(D):
                    x[i][d] += P[p + "fc2.b"][d] + sum(P[p + "fc2.W"][d][f] * a[f] for f in range(Fd))
        feats.append(ln(x[0], P["lnf.g"], P["lnf.b"]))
    Mh = cfg.mil_hidden
    a_ = []
    for h in feats:
        acc = 0.0
        for j in range(Mh):
            tv = math.tanh(P["mil.V.b"][j] + sum(P["mil.V.W"][j][d] * h[d] for d in range(D)))
            sv = 1.0 / (1.0 + math.exp(-(P["mil.U.b"][j] + sum(P["mil.U.W"][j][d] * h[d] for d in range(D)))))
            acc += P["mil.w"][j] * tv * sv
        a_.append(acc)
    mx = max(a_)
    ex = [math.exp(v - mx) for v in a_]
    alpha = [e / sum(ex) for e in ex]
    z = [sum(alpha[t_] * feats[t_][d] for t_ in range(n)) for d in range(D)]
    y = [P["head.b"][c] + sum(P["head.W"][c][d] * z[d] for d in range(D)) for c in range(cfg.n_classes)]
    if cfg.n_classes == 1:
        pr = 1.0 / (1.0 + math.exp(-y[0]))
        loss = -(label * math.log(pr) + (1 - label) * math.log(1 - pr))
    else:
        loss = -math.log(math.exp(y[label]) / sum(math.exp(v) for v in y))
    return loss, y, alpha, feats


@pytest.mark.parametrize("ncls,label", [(1, 1), (3, 2)])
def test_naive_scalar_forward(ncls, label):
    cfg = gen.SlideConfig(16, 8, 8, 2, 2, 2, 4, ncls)
    prm = gen.make_params(cfg, 11, perturbed=True, std=0.3)   # large weights: non-trivial softmaxes
    X = gen.make_pixels(cfg, 3, 12, kind="uniform").astype(np.float64)
    loss, y, alpha, feats = _naive_forward(cfg, prm, X, label)
    res = so.slide_step(prm, X, label, cfg)
    assert abs(res["loss"] - loss) < 1e-12
    np.testing.assert_allclose(res["logits"], y, atol=1e-12)
    np.testing.assert_allclose(res["alpha"], alpha, atol=1e-13)
    np.testing.assert_allclose(res["H"], np.array(feats), atol=1e-11)


# ---------------------------------------------------------------- closed forms, invariants

def test_pool_single_tile():
    cfg, prm, _, _ = _case("tiny")
    rng = np.random.default_rng(5)
    Hf = rng.standard_normal((1, cfg.dim))
    loss, y, alpha, z, c = so.pool_fwd(prm, Hf, 1, cfg)
    G, g = so.pool_bwd(c)
    assert alpha.tolist() == [1.0]
    np.testing.assert_allclose(z, Hf[0])
    dy = 1 / (1 + math.exp(-y[0])) - 1
    np.testing.assert_allclose(G[0], prm["head.W"][0].astype(np.float64) * dy, atol=1e-15)
    for k in ("mil.V.W", "mil.U.W", "mil.w", "mil.V.b", "mil.U.b"):
        assert np.abs(g[k]).max() < 1e-18


def test_pool_zero_attention_vector_is_mean_pool():
    cfg, prm, _, _ = _case("tiny")
    prm = dict(prm)
    prm["mil.w"] = np.zeros_like(prm["mil.w"])
    rng = np.random.default_rng(6)
    N = 13
    Hf = rng.standard_normal((N, cfg.dim))
    loss, y, alpha, z, c = so.pool_fwd(prm, Hf, 0, cfg)
    G, g = so.pool_bwd(c)
    np.testing.assert_allclose(alpha, np.full(N, 1.0 / N), atol=1e-16)
    np.testing.assert_allclose(z, Hf.mean(axis=0), atol=1e-15)
    dy = 1 / (1 + math.exp(-y[0]))
    Gref = np.tile(prm["head.W"][0].astype(np.float64) * dy / N, (N, 1))
    np.testing.assert_allclose(G, Gref, atol=1e-16)


def test_pool_softmax_properties_and_shift():
    cfg, prm, _, _ = _case("tiny", n_classes=4)
    rng = np.random.default_rng(7)
    Hf = rng.standard_normal((50, cfg.dim)) * 3
    loss, y, alpha, z, c = so.pool_fwd(prm, Hf, 2, cfg)
    assert abs(alpha.sum() - 1) < 1e-14 and (alpha > 0).all()
    # duplicate tiles get equal weights and equal gradient rows
    H2 = np.concatenate([Hf, Hf[:1]], axis=0)
    _, _, a2, _, c2 = so.pool_fwd(prm, H2, 2, cfg)
    G2, _ = so.pool_bwd(c2)
    assert a2[0] == a2[-1]
    np.testing.assert_allclose(G2[0], G2[-1], rtol=1e-13, atol=1e-18)


def test_pool_max_limit():
    cfg, prm, _, _ = _case("tiny")
    prm = {k: v.astype(np.float64) for k, v in prm.items()}
    prm["mil.w"] = prm["mil.w"] * 0 + 50.0
    prm["mil.V.W"] *= 0
    prm["mil.U.W"] *= 0
    prm["mil.U.b"] = prm["mil.U.b"] * 0 + 10.0
    # a_n = 50 * Mh * tanh(bV.) sigma(10): make tile 4 stand out through V bias? use V.W on one feature instead
    prm["mil.V.b"] *= 0
    prm["mil.V.W"][:, 0] = 1.0
    Hf = np.zeros((9, cfg.dim))
    Hf[:, 1:] = np.random.default_rng(8).standard_normal((9, cfg.dim - 1))
    Hf[4, 0] = 3.0
    _, _, alpha, z, _ = so.pool_fwd(prm, Hf, 0, cfg)
    assert alpha[4] > 1 - 1e-12
    np.testing.assert_allclose(z, Hf[4], atol=1e-9)


def test_loss_at_zero_logits():
    cfg, prm, _, _ = _case("tiny")
    prm = dict(prm)
    prm["head.W"] = np.zeros_like(prm["head.W"])
    prm["head.b"] = np.zeros_like(prm["head.b"])
    Hf = np.random.default_rng(9).standard_normal((5, cfg.dim))
    for label in (0, 1):
        loss, y, _, _, c = so.pool_fwd(prm, Hf, label, cfg)
        assert abs(loss - math.log(2)) < 1e-15 and abs(c["dy"][0] - (0.5 - label)) < 1e-15
    cfg4 = replace(cfg, n_classes=4)
    prm4 = gen.make_params(cfg4, 1)
    prm4["head.W"] *= 0
    loss, y, _, _, c = so.pool_fwd(prm4, Hf, 3, cfg4)
    assert abs(loss - math.log(4)) < 1e-15
    np.testing.assert_allclose(c["dy"], [0.25, 0.25, 0.25, -0.75], atol=1e-15)


def test_tile_permutation():
    cfg, prm, X, label = _case("tiny")
    perm = np.random.default_rng(10).permutation(X.shape[0])
    a = so.slide_step(prm, X, label, cfg)
    b = so.slide_step(prm, X[perm], label, cfg)
    assert abs(a["loss"] - b["loss"]) < 1e-14
    np.testing.assert_allclose(a["alpha"][perm], b["alpha"], atol=1e-15)
    np.testing.assert_allclose(a["G"][perm], b["G"], atol=1e-15)
    np.testing.assert_allclose(a["dX"][perm], b["dX"], atol=1e-15)
    for k in a["grads"]:
        np.testing.assert_allclose(a["grads"][k], b["grads"][k], atol=1e-13 * max(1.0, np.abs(a["grads"][k]).max()))


def test_chunk_additivity_and_mean_needs_factor():
    """Paper, Results 'Gradient Equivalence': chunks (encoder ranks) reproduce the one-device gradient
    when chunk gradients are summed; a mean over chunks needs the factor #chunks (Method, scaling remark)."""
    cfg, prm, X, label = _case("tiny")
    whole = so.slide_step(prm, X, label, cfg)
    chunks = [(0, 3), (3, 4), (4, 11), (11, 16)]
    part = so.slide_step(prm, X, label, cfg, chunks=chunks, keep_caches=False)
    for k in whole["grads"]:
        np.testing.assert_allclose(part["grads"][k], whole["grads"][k], rtol=0,
                                   atol=1e-12 * max(1e-3, np.abs(whole["grads"][k]).max()))
    np.testing.assert_allclose(part["dX"], whole["dX"], atol=1e-16)
    # equal-size chunks, encoder gradients averaged: off by exactly the number of chunks
    eq = [(0, 4), (4, 8), (8, 12), (12, 16)]
    feats = [so.encoder_fwd(prm, X[lo:hi], cfg) for lo, hi in eq]
    Hf = np.concatenate([f[0] for f in feats])
    _, _, _, _, pc = so.pool_fwd(prm, Hf, label, cfg)
    G, _ = so.pool_bwd(pc)
    mean = None
    for (lo, hi), (_, cache) in zip(eq, feats):
        ge, _ = so.encoder_bwd(cache, G[lo:hi], cfg, False)
        mean = ge if mean is None else {k: mean[k] + ge[k] for k in ge}
    k = "l0.fc1.W"
    np.testing.assert_allclose(mean[k] / len(eq) * len(eq), whole["grads"][k], atol=1e-15)
    assert np.abs(mean[k] / len(eq) - whole["grads"][k]).max() > 0.5 * np.abs(whole["grads"][k]).max()


def test_key_bias_gradient_is_zero():
    cfg, prm, X, label = _case("tiny")
    res = so.slide_step(prm, X, label, cfg)
    D = cfg.dim
    for l in range(cfg.layers):
        g = res["grads"][f"l{l}.qkv.b"]
        assert np.abs(g[D:2 * D]).max() <= 1e-12 * np.abs(g).max()


def test_depth_zero_encoder():
    cfg = gen.SlideConfig(32, 8, 64, 0, 2, 4, 32, 1)
    prm = gen.make_params(cfg, 3, perturbed=True)
    X = gen.make_pixels(cfg, 6, 4, kind="uniform").astype(np.float64)
    res = so.slide_step(prm, X, 1, cfg)
    np.testing.assert_allclose(res["alpha"], 1 / 6, atol=1e-15)
    assert np.abs(res["dX"]).max() == 0 and np.abs(res["grads"]["pe.W"]).max() == 0


def test_identity_blocks():
    cfg, prm, X, label = _case("tiny")
    prm = {k: v.astype(np.float64) for k, v in prm.items()}
    for l in range(cfg.layers):
        for k in ("proj.W", "proj.b", "fc2.W", "fc2.b"):
            prm[f"l{l}.{k}"] *= 0
    Hf, _ = so.encoder_fwd(prm, X, cfg)
    x0 = prm["cls"] + prm["pos"][0]
    mu, var = x0.mean(), x0.var()
    ref = (x0 - mu) / np.sqrt(var + cfg.ln_eps) * prm["lnf.g"] + prm["lnf.b"]
    np.testing.assert_allclose(Hf, np.tile(ref, (X.shape[0], 1)), atol=1e-14)


def test_layernorm_properties():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((7, 64)) * 2 + 1
    g, b = rng.standard_normal(64), rng.standard_normal(64)
    y, cache = so._ln_fwd(x, g, b, 1e-6)
    xh = cache[0]
    np.testing.assert_allclose(xh.mean(-1), 0, atol=1e-15)
    np.testing.assert_allclose(xh.var(-1), 1 / (1 + 1e-6 / x.var(-1)), rtol=1e-12)
    y2, _ = so._ln_fwd(3.0 * x + 5.0, g, b, 9e-6)       # affine invariance (eps scales with a^2)
    np.testing.assert_allclose(y2, y, atol=1e-12)
    dx, _, _ = so._ln_bwd(rng.standard_normal((7, 64)), g, cache)
    np.testing.assert_allclose(dx.sum(-1), 0, atol=1e-13)


def test_gelu_matches_normal_cdf_form():
    from scipy.stats import norm
    m = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(so._gelu(m), m * norm.cdf(m), atol=1e-15)
    np.testing.assert_allclose(so._gelu_grad(m), norm.cdf(m) + m * norm.pdf(m), atol=1e-15)


def test_patch_order():
    cfg = gen.SlideConfig(32, 8, 8, 0, 1, 2, 4, 1)
    X = np.arange(2 * 3 * 32 * 32, dtype=np.float64).reshape(2, 3, 32, 32)
    p = so.patchify(X, cfg)
    # patch (gy=2, gx=3) of tile 1, element (c=1, py=5, px=6)
    assert p[1, 2 * 4 + 3, 1 * 64 + 5 * 8 + 6] == X[1, 1, 2 * 8 + 5, 3 * 8 + 6]
    np.testing.assert_array_equal(so.unpatchify(p, cfg), X)
