"""Test-side glue for the convolutional tile encoder: seeded generators, the ctypes binding, the CPU oracle."""
from __future__ import annotations

import numpy as np

import gen
from slide_harness import rel_l2


def resnet_inputs(name, n=None, n_classes=None, tile=None):
    """(cfg, params on the bf16 grid where the library rounds them, pixels on the bf16 grid, label)."""
    from dataclasses import replace
    cfg, n0 = gen.RESNET_CONFIGS[name]
    if n_classes:
        cfg = replace(cfg, n_classes=n_classes)
    if tile:
        cfg = replace(cfg, tile=tile)
    ds, ws, ls = gen.RESNET_SEEDS[name]
    n = n or n0
    prm = gen.make_resnet_params(cfg, ws)
    # convolution weights are used as bf16 by the library: start both sides from the same numbers
    prm = {k: (gen.to_bf16_grid(v) if k.endswith("conv.W") or ".conv" in k else v) for k, v in prm.items()}
    X = gen.to_bf16_grid(gen.make_pixels(cfg, n, ds, kind="blur"))
    rng = np.random.Generator(np.random.PCG64(ls))
    label = int(rng.random() < 0.5) if cfg.n_classes == 1 else int(rng.integers(0, cfg.n_classes))
    return cfg, prm, X, label


class GpuResNet:
    """A bound resnet_ctx on cuda:0 with flat parameter / gradient vectors."""

    def __init__(self, cfg, prm: dict, n_tiles: int, arena_bytes: int | None = None):
        import torch
        from paper_2403_04865_amd import ResNetLib, resnet_config_from
        self.torch = torch
        self.cfg = cfg
        self.dev = torch.device("cuda:0")
        self.lib = ResNetLib(resnet_config_from(cfg))
        self.layout = self.lib.param_layout()
        shapes = dict(gen.resnet_param_shapes(cfg))
        assert [n for n, _, _ in self.layout] == [n for n, _ in gen.resnet_param_shapes(cfg)]
        flat = np.zeros(self.lib.resnet_param_count(), dtype=np.float32)
        for name, off, ln in self.layout:
            assert int(np.prod(shapes[name])) == ln, name
            flat[off:off + ln] = np.asarray(prm[name], dtype=np.float32).reshape(-1)
        self.shapes = shapes
        self.params = torch.from_numpy(flat).to(self.dev)
        self.grads = torch.zeros_like(self.params)
        nbytes = self.lib.resnet_arena_bytes(n_tiles) if arena_bytes is None else arena_bytes
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.arena.data_ptr()) % 256
        self.arena = self.arena[off:off + nbytes]
        self.lib.resnet_bind(self.params, self.grads, self.arena)

    def to_dev(self, x):
        return self.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.dev).to(self.torch.bfloat16).contiguous()

    def grads_dict(self):
        g = self.grads.cpu().numpy()
        return {name: g[off:off + ln].reshape(self.shapes[name]).astype(np.float64) for name, off, ln in self.layout}

    def view(self, ptr, shape):
        torch = self.torch
        off = ptr - self.arena.data_ptr()
        n = int(np.prod(shape)) * 4
        return self.arena[off:off + n].view(torch.float32).reshape(shape).cpu().numpy().astype(np.float64)

    def activations(self):
        """The saved activations of the last forward as float64 [n, C, side, side] arrays, in the library's order."""
        torch = self.torch
        out = []
        for i in range(self.lib.resnet_saved_activations()):
            ptr, side, ch = self.lib.resnet_saved_activation(i)
            off = ptr - self.arena.data_ptr()
            nb = self.n_last * side * side * ch * 2
            t = self.arena[off:off + nb].view(torch.bfloat16).reshape(self.n_last, side, side, ch)
            out.append(t.float().cpu().numpy().transpose(0, 3, 1, 2).astype(np.float64))
        return out

    def step(self, X, label, accumulate=False):
        torch = self.torch
        N = X.shape[0]
        self.n_last = N
        px = X if isinstance(X, torch.Tensor) else self.to_dev(X)
        loss = torch.zeros(1, device=self.dev)
        logits = torch.zeros(self.cfg.n_classes, device=self.dev)
        alpha = torch.zeros(N, device=self.dev)
        self.lib.resnet_slide_step_fwd(px, N, label, loss, logits, alpha)
        H = self.view(self.lib.resnet_features(), (N, self.cfg.dim))
        self.lib.resnet_slide_step_bwd(accumulate)
        torch.cuda.synchronize()
        G = self.view(self.lib.resnet_feature_grads(), (N, self.cfg.dim))
        return {"loss": float(loss.item()), "logits": logits.cpu().numpy().astype(np.float64),
                "alpha": alpha.cpu().numpy().astype(np.float64), "H": H, "G": G, "grads": self.grads_dict()}


def bf16_store(a):
    """Round to the nearest bfloat16 (ties to even): the precision in which the library stores activations."""
    return gen.to_bf16_grid(a.astype(np.float32)).astype(np.float64)


def compare_resnet_step(gpu, ref, tol, grads=True):
    """Relative L2 of loss, logits, attention weights, features, feature gradients and every parameter gradient."""
    errs = {"loss": abs(gpu["loss"] - ref["loss"]) / max(abs(ref["loss"]), 1e-12)}
    for k in ("logits", "alpha", "H") + (("G",) if grads else ()):
        errs[k] = rel_l2(gpu[k], ref[k])
    if grads:
        for name, g in ref["grads"].items():
            errs[name] = rel_l2(gpu["grads"][name], g)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    return errs, bad


def replay_reference(gpu: 'GpuResNet', prm, X, label):
    """The oracle's step with every ReLU mask and pooling maximum decided on the numbers the library decided them on.

    A ReLU network's gradient is discontinuous where a pre-activation crosses zero, so two correct 16-bit computations
    of the forward (which agree to the storage rounding, a few 1e-3) give gradients that differ wherever one of them
    has a stored activation at zero and the other does not.  The oracle therefore takes each stored activation from
    the library at the point where the library stored it (its `store` argument) and computes everything else itself
    in float64: each layer's forward from the library's previous stored tensor (returned per storage point as `links`:
    relative L2 between what the library stored and the oracle's unrounded value), the normalisation statistics, the
    aggregator, and the whole backward.  Returns (reference dict, links, max-pooling output of the library).
    """
    from oracle import resnet_oracle as ro
    acts = gpu.activations()
    pooled = acts.pop(2)
    it = iter(acts)
    links = []

    def replay(a):
        g = next(it)
        assert g.shape == a.shape, (g.shape, a.shape)
        links.append(rel_l2(g, a))
        return g

    ref = ro.slide_step({k: np.asarray(v, dtype=np.float64) for k, v in prm.items()}, np.asarray(X, dtype=np.float64),
                        label, gpu.cfg, store=replay)
    assert next(it, None) is None
    return ref, links, (pooled, ro.maxpool_fwd(acts[1])[0])
