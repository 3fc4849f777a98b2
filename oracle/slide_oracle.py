"""CPU oracle for one end-to-end slide training step.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain reference that the HIP path is checked against.
Only tests, the smoke check and the bench's cpu_baseline leg may import it; the
product path never does.  It shares no code with the HIP path.

What it computes (paper, Method + appendix listing): every tile of a slide goes
through a tile encoder, the feature matrix goes through a gated-attention MIL
aggregator that yields class logits, a slide-level criterion gives one scalar
loss, and that loss is differentiated with respect to every encoder and
aggregator parameter and the pixels.  The method is exact (the paper's Results,
"Gradient Equivalence", claims equality with the one-device gradient), so the
oracle is the definition written out: forward of the composed function, then
reverse-mode derivatives step by step, in float64, with library matmul as the
only primitive.  No blocking, fusion or reordering.

The paper fixes the scheme (encoder -> gather -> aggregator -> loss -> feature
gradients -> scatter -> pseudo-loss backward) but not the encoder's internals;
those follow the workload definitions: a pre-LayerNorm vision transformer with
a learned CLS token and position table, biases on all linear maps, exact (erf)
GELU, softmax attention scaled by 1/sqrt(d_h), a final LayerNorm on the CLS
row; the aggregator is the gated attention of Ilse et al. (cited in Method):
a_n = w.(tanh(V h_n + b_V) * sigmoid(U h_n + b_U)), softmax over tiles,
z = sum_n alpha_n h_n, logits = W_c z + b_c.

Parity pins: every function here is pinned by tests/test_oracle_*.py (finite
differences of the whole scalar loss, a second brute-force implementation, an
independent autograd graph of library routines, closed-form special cases and
invariants).  Nothing is "parity unpinned".

Parameters are a dict name -> ndarray (names: pe.W, pe.b, cls, pos, l{i}.ln1.g,
l{i}.ln1.b, l{i}.qkv.W, l{i}.qkv.b, l{i}.proj.W, l{i}.proj.b, l{i}.ln2.g,
l{i}.ln2.b, l{i}.fc1.W, l{i}.fc1.b, l{i}.fc2.W, l{i}.fc2.b, lnf.g, lnf.b,
mil.V.W, mil.V.b, mil.U.W, mil.U.b, mil.w, head.W, head.b); W is [out][in].
`cfg` is any object with fields tile, patch, dim, layers, heads, mlp_ratio,
mil_hidden, n_classes, ln_eps.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------

def _ln_fwd(x, g, b, eps):
    """LayerNorm over the last axis, biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    return xh * g + b, (xh, rstd)


def _ln_bwd(dy, g, cache):
    xh, rstd = cache
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True)
                 - xh * (dxh * xh).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xh).sum(axis=red), dy.sum(axis=red)


def _gelu(m):
    return 0.5 * m * (1.0 + erf(m / np.sqrt(2.0)))


def _gelu_grad(m):
    return 0.5 * (1.0 + erf(m / np.sqrt(2.0))) + m * np.exp(-0.5 * m * m) / np.sqrt(2.0 * np.pi)


def _softmax_last(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def _rows(a):
    """View [..., C] as a 2-D [rows, C] matrix (all leading axes are summed by `.T @`)."""
    return a.reshape(-1, a.shape[-1])


def patchify(X, cfg):
    """[n,3,S,S] -> [n, g*g, 3*P*P]; patches in (gy, gx) order, flattened (c, py, px)."""
    n = X.shape[0]
    P, g = cfg.patch, cfg.tile // cfg.patch
    p = X.reshape(n, 3, g, P, g, P)           # n c gy py gx px
    p = p.transpose(0, 2, 4, 1, 3, 5)         # n gy gx c py px
    return p.reshape(n, g * g, 3 * P * P)


def unpatchify(dp, cfg):
    """Inverse index map of `patchify` (used for the pixel gradient)."""
    n = dp.shape[0]
    P, g = cfg.patch, cfg.tile // cfg.patch
    d = dp.reshape(n, g, g, 3, P, P).transpose(0, 3, 1, 4, 2, 5)
    return d.reshape(n, 3, g * P, g * P)


# ----------------------------------------------------------------------------
# tile encoder (paper, appendix listing: the encoder ranks' forward step)
# ----------------------------------------------------------------------------

def encoder_fwd(prm, X, cfg, dtype=np.float64):
    """Tile pixels [n,3,S,S] -> CLS features [n,D] and a cache for the backward."""
    P = {k: np.asarray(v, dtype=dtype) for k, v in prm.items()}
    X = np.asarray(X, dtype=dtype)
    n = X.shape[0]
    D, H = cfg.dim, cfg.heads
    dh = D // H
    T = (cfg.tile // cfg.patch) ** 2 + 1
    pt = patchify(X, cfg)
    x = np.empty((n, T, D), dtype=dtype)
    x[:, 1:, :] = pt @ P["pe.W"].T + P["pe.b"] + P["pos"][1:]
    x[:, 0, :] = P["cls"] + P["pos"][0]
    layers = []
    for l in range(cfg.layers):
        p = f"l{l}."
        c = {"x_in": x}
        u, c["ln1"] = _ln_fwd(x, P[p + "ln1.g"], P[p + "ln1.b"], cfg.ln_eps)
        qkv = u @ P[p + "qkv.W"].T + P[p + "qkv.b"]
        q = qkv[..., 0 * D:1 * D].reshape(n, T, H, dh).transpose(0, 2, 1, 3)
        k = qkv[..., 1 * D:2 * D].reshape(n, T, H, dh).transpose(0, 2, 1, 3)
        v = qkv[..., 2 * D:3 * D].reshape(n, T, H, dh).transpose(0, 2, 1, 3)
        S = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(dh)
        Pr = _softmax_last(S)
        o = (Pr @ v).transpose(0, 2, 1, 3).reshape(n, T, D)
        x = x + o @ P[p + "proj.W"].T + P[p + "proj.b"]
        c.update(u=u, q=q, k=k, v=v, Pr=Pr, o=o)
        u2, c["ln2"] = _ln_fwd(x, P[p + "ln2.g"], P[p + "ln2.b"], cfg.ln_eps)
        m = u2 @ P[p + "fc1.W"].T + P[p + "fc1.b"]
        a = _gelu(m)
        x = x + a @ P[p + "fc2.W"].T + P[p + "fc2.b"]
        c.update(u2=u2, m=m, a=a)
        layers.append(c)
    h, lnf = _ln_fwd(x[:, 0, :], P["lnf.g"], P["lnf.b"], cfg.ln_eps)
    return h, {"P": P, "patches": pt, "layers": layers, "lnf": lnf, "n": n, "T": T}


def encoder_bwd(cache, G, cfg, want_pixel_grad=True):
    """Backward of the encoder with upstream feature gradient G [n,D].

    This is the gradient of the paper's pseudo-loss sum_{tiles,features} f*g
    (Method, inline equation; appendix listing, the encoder ranks' backward step) with
    no rank factor: on one device the encoder gradient is J^T g as is.
    Returns (dict of parameter gradients, pixel gradient or None).
    """
    P, n, T = cache["P"], cache["n"], cache["T"]
    D, H = cfg.dim, cfg.heads
    dh = D // H
    dt = G.dtype
    g = {}
    dh_cls, g["lnf.g"], g["lnf.b"] = _ln_bwd(np.asarray(G), P["lnf.g"], cache["lnf"])
    dx = np.zeros((n, T, D), dtype=dt)
    dx[:, 0, :] = dh_cls
    for l in reversed(range(cfg.layers)):
        p = f"l{l}."
        c = cache["layers"][l]
        # x_out = x_mid + gelu(LN2(x_mid) W1^T + b1) W2^T + b2
        g[p + "fc2.b"] = dx.sum(axis=(0, 1))
        g[p + "fc2.W"] = _rows(dx).T @ _rows(c["a"])
        da = dx @ P[p + "fc2.W"]
        dm = da * _gelu_grad(c["m"])
        g[p + "fc1.b"] = dm.sum(axis=(0, 1))
        g[p + "fc1.W"] = _rows(dm).T @ _rows(c["u2"])
        du2 = dm @ P[p + "fc1.W"]
        dxm, g[p + "ln2.g"], g[p + "ln2.b"] = _ln_bwd(du2, P[p + "ln2.g"], c["ln2"])
        dx = dx + dxm
        # x_mid = x_in + attn(LN1(x_in)) Wo^T + bo
        g[p + "proj.b"] = dx.sum(axis=(0, 1))
        g[p + "proj.W"] = _rows(dx).T @ _rows(c["o"])
        do = (dx @ P[p + "proj.W"]).reshape(n, T, H, dh).transpose(0, 2, 1, 3)
        dv = c["Pr"].transpose(0, 1, 3, 2) @ do
        dP = do @ c["v"].transpose(0, 1, 3, 2)
        dS = c["Pr"] * (dP - (dP * c["Pr"]).sum(axis=-1, keepdims=True))
        dq = (dS @ c["k"]) / np.sqrt(dh)
        dk = (dS.transpose(0, 1, 3, 2) @ c["q"]) / np.sqrt(dh)
        dqkv = np.concatenate(
            [t.transpose(0, 2, 1, 3).reshape(n, T, D) for t in (dq, dk, dv)], axis=-1)
        g[p + "qkv.b"] = dqkv.sum(axis=(0, 1))
        g[p + "qkv.W"] = _rows(dqkv).T @ _rows(c["u"])
        du = dqkv @ P[p + "qkv.W"]
        dxi, g[p + "ln1.g"], g[p + "ln1.b"] = _ln_bwd(du, P[p + "ln1.g"], c["ln1"])
        dx = dx + dxi
    g["pos"] = dx.sum(axis=0)
    g["cls"] = dx[:, 0, :].sum(axis=0)
    dtok = dx[:, 1:, :]
    g["pe.b"] = dtok.sum(axis=(0, 1))
    g["pe.W"] = _rows(dtok).T @ _rows(cache["patches"])
    dX = unpatchify(dtok @ P["pe.W"], cfg) if want_pixel_grad else None
    return g, dX


# ----------------------------------------------------------------------------
# aggregator + criterion (paper, appendix listing: the aggregator rank's forward, criterion and
# backward to the gathered features; Method, paragraph on the aggregator)
# ----------------------------------------------------------------------------

def pool_fwd(prm, Hf, label, cfg, dtype=np.float64):
    """Gated-attention MIL pooling, class logits and the slide loss."""
    P = {k: np.asarray(v, dtype=dtype) for k, v in prm.items() if k.startswith(("mil.", "head."))}
    Hf = np.asarray(Hf, dtype=dtype)
    t = np.tanh(Hf @ P["mil.V.W"].T + P["mil.V.b"])
    s = 1.0 / (1.0 + np.exp(-(Hf @ P["mil.U.W"].T + P["mil.U.b"])))
    a = (t * s) @ P["mil.w"]
    alpha = _softmax_last(a)
    z = alpha @ Hf
    y = P["head.W"] @ z + P["head.b"]
    if cfg.n_classes == 1:
        # binary cross-entropy on one logit, stable form
        loss = max(y[0], 0.0) - y[0] * label + np.log1p(np.exp(-abs(y[0])))
        dy = np.array([1.0 / (1.0 + np.exp(-y[0])) - label], dtype=dtype)
    else:
        ym = y.max()
        lse = ym + np.log(np.exp(y - ym).sum())
        loss = lse - y[label]
        dy = np.exp(y - lse)
        dy[label] -= 1.0
    cache = {"P": P, "H": Hf, "t": t, "s": s, "alpha": alpha, "z": z, "dy": dy}
    return float(loss), y, alpha, z, cache


def pool_bwd(cache):
    """Feature-gradient matrix G [N,D] and the aggregator's parameter gradients."""
    P, Hf, t, s, alpha, z, dy = (cache[k] for k in ("P", "H", "t", "s", "alpha", "z", "dy"))
    g = {}
    g["head.W"] = np.outer(dy, z)
    g["head.b"] = dy.copy()
    dz = P["head.W"].T @ dy
    r = Hf @ dz
    da = alpha * (r - alpha @ r)                 # softmax backward
    g["mil.w"] = da @ (t * s)
    dgate = da[:, None] * P["mil.w"][None, :]    # d(t*s)
    dpV = dgate * s * (1.0 - t * t)
    dpU = dgate * t * s * (1.0 - s)
    g["mil.V.W"] = dpV.T @ Hf
    g["mil.V.b"] = dpV.sum(axis=0)
    g["mil.U.W"] = dpU.T @ Hf
    g["mil.U.b"] = dpU.sum(axis=0)
    G = alpha[:, None] * dz[None, :] + dpV @ P["mil.V.W"] + dpU @ P["mil.U.W"]
    return G, g


# ----------------------------------------------------------------------------
# whole step
# ----------------------------------------------------------------------------

def slide_loss(prm, X, label, cfg, dtype=np.float64):
    """Forward only: the scalar slide loss (used by finite-difference pins)."""
    Hf, _ = encoder_fwd(prm, X, cfg, dtype)
    return pool_fwd(prm, Hf, label, cfg, dtype)[0]


def slide_step(prm, X, label, cfg, chunks=None, want_pixel_grad=True, dtype=np.float64,
               keep_caches=True):
    """One forward + backward step over all tiles of a slide.

    chunks=None: the one-device definition: encode all tiles, aggregate, loss,
    backward through aggregator and encoder.
    chunks=[(lo,hi),...]: the paper's scheme with "encoder rank" read as "tile
    chunk": encode each chunk, concatenate features (gather), aggregator forward
    and backward on the full matrix, route rows of G back to their chunk
    (scatter), back-propagate each chunk's pseudo-loss, and SUM the encoder
    gradients over chunks (the listing's factor world_size-1 only undoes the
    gradient *mean* of its data-parallel wrapper; a sum needs none).
    keep_caches=False drops each chunk's saved activations after its features
    are taken and runs that chunk's forward again just before its backward
    (same numbers, bounded memory).
    Returns dict(loss, logits, alpha, z, H, G, grads, dX).
    """
    X = np.asarray(X)
    N = X.shape[0]
    if chunks is None:
        chunks = [(0, N)]
    feats = []
    for lo, hi in chunks:
        h, cache = encoder_fwd(prm, X[lo:hi], cfg, dtype)
        feats.append((h, cache if keep_caches else None))
    Hf = np.concatenate([f[0] for f in feats], axis=0)
    loss, y, alpha, z, pc = pool_fwd(prm, Hf, label, cfg, dtype)
    G, grads = pool_bwd(pc)
    dX = np.zeros(X.shape, dtype=dtype) if want_pixel_grad else None
    row = 0
    for (lo, hi), (_, cache) in zip(chunks, feats):
        if cache is None:
            cache = encoder_fwd(prm, X[lo:hi], cfg, dtype)[1]
        ge, dXc = encoder_bwd(cache, G[row:row + (hi - lo)], cfg, want_pixel_grad)
        row += hi - lo
        for k, v in ge.items():
            grads[k] = grads[k] + v if k in grads else v
        if want_pixel_grad:
            dX[lo:hi] = dXc
    return {"loss": loss, "logits": y, "alpha": alpha, "z": z, "H": Hf, "G": G,
            "grads": grads, "dX": dX}
