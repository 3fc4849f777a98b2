"""Seeded synthetic slides, weights and labels.

The paper's slides are private clinical data (Results: EGFR / breast cohorts);
these generators reproduce only their *shape*: a bag of N RGB tiles of 224 px
(Results, whole-slide breast experiment), thousands to tens of thousands of
tiles per slide (Method, Fig. 1c).  Tiles are i.i.d. because tiles interact
only through the permutation-invariant aggregator (Method, paragraph on the
gather step).

Everything here is input plumbing: shapes, names and RNG recipes.  No encoder,
pool, loss or gradient arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np


@dataclass(frozen=True)
class SlideConfig:
    tile: int        # S: tile side in pixels
    patch: int       # P: patch side
    dim: int         # D: encoder width
    layers: int      # L
    heads: int       # H
    mlp_ratio: int   # F = mlp_ratio * D
    mil_hidden: int  # M_h: gated-attention hidden width
    n_classes: int   # C: 1 -> one logit + BCE, >1 -> softmax cross-entropy
    ln_eps: float = 1e-6

    @property
    def grid(self) -> int:
        return self.tile // self.patch

    @property
    def tokens(self) -> int:  # T = patches + CLS
        return self.grid * self.grid + 1

    @property
    def patch_dim(self) -> int:
        return 3 * self.patch * self.patch

    @property
    def ffn(self) -> int:
        return self.mlp_ratio * self.dim

    def as_dict(self):
        return asdict(self)


# Workloads (name -> (config, n_tiles)).  "probe" is a brute-force-sized case.
CONFIGS = {
    "probe":  (SlideConfig(16, 8, 8, 1, 1, 2, 4, 1), 3),
    "tiny":   (SlideConfig(32, 8, 64, 2, 2, 4, 32, 1), 16),
    "small":  (SlideConfig(224, 16, 384, 12, 6, 4, 128, 1), 256),
    "medium": (SlideConfig(224, 16, 384, 12, 6, 4, 128, 1), 2048),
    "large":  (SlideConfig(224, 16, 384, 12, 6, 4, 256, 4), 8192),
    "full":   (SlideConfig(224, 16, 768, 12, 12, 4, 256, 1), 16384),
}

# (data, weights, label) seeds per workload.
SEEDS = {
    "probe":  (1000, 2000, 3000),
    "tiny":   (1001, 2001, 3001),
    "small":  (1002, 2002, 3002),
    "medium": (1003, 2002, 3003),
    "large":  (1004, 2002, 3004),
    "full":   (1005, 2005, 3005),
}


def param_shapes(cfg: SlideConfig):
    """Ordered (name, shape) list of every trainable tensor.  W is [out][in]."""
    D, F, T, Mh, C = cfg.dim, cfg.ffn, cfg.tokens, cfg.mil_hidden, cfg.n_classes
    out = [("pe.W", (D, cfg.patch_dim)), ("pe.b", (D,)), ("cls", (D,)), ("pos", (T, D))]
    for l in range(cfg.layers):
        p = f"l{l}."
        out += [
            (p + "ln1.g", (D,)), (p + "ln1.b", (D,)),
            (p + "qkv.W", (3 * D, D)), (p + "qkv.b", (3 * D,)),
            (p + "proj.W", (D, D)), (p + "proj.b", (D,)),
            (p + "ln2.g", (D,)), (p + "ln2.b", (D,)),
            (p + "fc1.W", (F, D)), (p + "fc1.b", (F,)),
            (p + "fc2.W", (D, F)), (p + "fc2.b", (D,)),
        ]
    out += [
        ("lnf.g", (D,)), ("lnf.b", (D,)),
        ("mil.V.W", (Mh, D)), ("mil.V.b", (Mh,)),
        ("mil.U.W", (Mh, D)), ("mil.U.b", (Mh,)),
        ("mil.w", (Mh,)),
        ("head.W", (C, D)), ("head.b", (C,)),
    ]
    return out


def _trunc_normal(rng, shape, std):
    """N(0, std^2) with draws outside +-2 std redrawn."""
    x = rng.standard_normal(shape)
    bad = np.abs(x) > 2.0
    while bad.any():
        x[bad] = rng.standard_normal(int(bad.sum()))
        bad = np.abs(x) > 2.0
    return x * std


def make_params(cfg: SlideConfig, seed: int, perturbed: bool = False, std: float = 0.02):
    """dict name -> float32 array.

    Plain init: every matrix, `cls`, `pos`, `mil.w` ~ truncated normal(std);
    biases 0, LayerNorm gain 1, shift 0.  `perturbed=True` also draws biases and
    shifts from the same law and sets gains to 1 + draw, so that a test cannot
    pass with a bias or gain term dropped.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, shape in param_shapes(cfg):
        leaf = name.split(".")[-1]
        is_gain = leaf == "g"
        is_shift = leaf == "b"
        if is_gain:
            v = np.ones(shape)
            if perturbed:
                v = v + _trunc_normal(rng, shape, std)
        elif is_shift:
            v = _trunc_normal(rng, shape, std) if perturbed else np.zeros(shape)
        else:
            v = _trunc_normal(rng, shape, std)
        out[name] = v.astype(np.float32)
    return out


def _box_blur5(x):
    """5x5 box mean over the last two axes, edge-replicated (separable shifted sums)."""
    S = x.shape[-1]
    p = np.pad(x, [(0, 0)] * (x.ndim - 2) + [(2, 2), (2, 2)], mode="edge")
    h = p[..., 0:S] + p[..., 1:S + 1] + p[..., 2:S + 2] + p[..., 3:S + 3] + p[..., 4:S + 4]
    v = h[..., 0:S, :] + h[..., 1:S + 1, :] + h[..., 2:S + 2, :] + h[..., 3:S + 3, :] + h[..., 4:S + 4, :]
    return v / np.float32(25.0)


def _pixel_chunk(S, seed, c, chunk, kind):
    rng = np.random.Generator(np.random.PCG64([seed, c]))
    if kind == "uniform":
        u = rng.random((chunk, 3, S, S), dtype=np.float32)
        return (u - np.float32(0.5)) / np.float32(0.25)
    if kind == "blur":
        g = rng.standard_normal((chunk, 3, S, S), dtype=np.float32)
        b = _box_blur5(g)
        return (np.clip(np.float32(0.5) + np.float32(1.25) * b, 0.0, 1.0) - np.float32(0.5)) / np.float32(0.25)
    raise ValueError(kind)


def make_pixels(cfg: SlideConfig, n_tiles: int, seed: int, kind: str = "blur",
                first_tile: int = 0, chunk: int = 64, workers: int = 1):
    """Normalised tile pixels, float32 [n_tiles, 3, S, S].

    kind="uniform": u ~ U[0,1), x = (u - 0.5) / 0.25.
    kind="blur":    g ~ N(0,1) i.i.d.; b = 5x5 box blur (std 0.2);
                    x01 = clip(0.5 + 1.25 b, 0, 1); x = (x01 - 0.5) / 0.25.
    Tiles are drawn in independent chunks of `chunk` tiles, chunk c from the
    stream PCG64([seed, c]), so any tile range can be produced on its own and
    chunks can be drawn by `workers` threads without changing the values.
    """
    S = cfg.tile
    out = np.empty((n_tiles, 3, S, S), dtype=np.float32)
    end = first_tile + n_tiles
    chunks = list(range(first_tile // chunk, (end + chunk - 1) // chunk)) if n_tiles > 0 else []

    def fill(c):
        x = _pixel_chunk(S, seed, c, chunk, kind)
        lo = c * chunk
        a = max(first_tile, lo)
        b = min(end, lo + chunk)
        out[a - first_tile: b - first_tile] = x[a - lo: b - lo]

    if workers > 1 and len(chunks) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, chunks))
    else:
        for c in chunks:
            fill(c)
    return out


def make_features(cfg: SlideConfig, n_rows: int, seed: int, spread: float = 0.25):
    """Synthetic [n_rows, D] tile-feature matrix with the statistics of final-LayerNorm CLS rows: a
    common component shared by all tiles plus a per-tile component (spread = their ratio, so that
    |H| / |H - mean row| is about 1 / spread), float32."""
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    mu = rng.standard_normal(cfg.dim)
    out = np.empty((n_rows, cfg.dim), dtype=np.float32)
    step = 65536
    for lo in range(0, n_rows, step):
        hi = min(n_rows, lo + step)
        out[lo:hi] = mu + spread * rng.standard_normal((hi - lo, cfg.dim))
    return out


def make_label(cfg: SlideConfig, seed: int) -> int:
    rng = np.random.Generator(np.random.PCG64(seed))
    if cfg.n_classes == 1:
        return int(rng.random() < 0.5)
    return int(rng.integers(0, cfg.n_classes))


def to_bf16_grid(x):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32.

    Used to make inputs and weights exactly representable in bfloat16, so the
    CPU oracle and the bf16 HIP path start from identical numbers.
    """
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)
