"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
from dataclasses import replace

import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4   # relative L2, fp32 path
BF16_TOL = 2e-2   # relative L2 on loss and parameter gradients, bf16 path


def _inputs(name, n=None, perturbed=True, n_classes=None, bf16=False, std=0.02):
    cfg, n0 = gen.CONFIGS[name]
    if n_classes:
        cfg = replace(cfg, n_classes=n_classes)
    ds, ws, ls = gen.SEEDS[name]
    n = n or n0
    prm = gen.make_params(cfg, ws, perturbed=perturbed, std=std)
    X = gen.make_pixels(cfg, n, ds, kind="uniform" if name in ("probe", "tiny") else "blur")
    if bf16:
        prm = {k: gen.to_bf16_grid(v) for k, v in prm.items()}
        X = gen.to_bf16_grid(X)
    return cfg, prm, X, gen.make_label(cfg, ls)


def _run(cfg, prm, X, label, dtype, tol, grad_tol=None, recompute=0):
    from oracle import slide_oracle as so
    from slide_harness import GpuSlide, compare_step
    print(f"case cfg={cfg} n={X.shape[0]} dtype={dtype} label={label} recompute={recompute}", flush=True)
    g = GpuSlide(cfg, prm, dtype, X.shape[0], recompute)
    out = g.step(X, label)
    ref = so.slide_step(prm, X.astype(np.float64), label, cfg)
    _, pool_same = so.pool_bwd(so.pool_fwd(prm, out["H"], label, cfg)[4])
    errs, bad, kappa = compare_step(out, ref, tol, cfg, grad_tol, pool_same)
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:8]
    print(f"kappa={kappa:.1f} worst:", worst, flush=True)
    assert not bad, bad
    return errs


@pytest.mark.parametrize("ncls,label", [(1, None), (4, 2)])
def test_tiny_fp32(ncls, label):
    cfg, prm, X, lab = _inputs("tiny", n_classes=ncls)
    _run(cfg, prm, X, lab if label is None else label, 0, FP32_TOL)


def test_tiny_fp32_ragged():
    # 13 tiles: row counts that are no multiple of any kernel tile
    cfg, prm, X, lab = _inputs("tiny", n=13, std=0.05)
    _run(cfg, prm, X, lab, 0, FP32_TOL)


def test_probe_fp32():
    cfg, prm, X, lab = _inputs("probe", std=0.2)
    _run(cfg, prm, X, lab, 0, FP32_TOL)


def test_tiny_bf16():
    cfg, prm, X, lab = _inputs("tiny", bf16=True)
    _run(cfg, prm, X, lab, 1, BF16_TOL)


def test_vit_s_fp32_21_tiles():
    # ViT-S/16 shapes (197 tokens, 6 heads of 64), 21 tiles: M = 4137 rows spans many GEMM tiles + a ragged tail
    cfg, prm, X, lab = _inputs("small", n=21)
    _run(cfg, prm, X, lab, 0, FP32_TOL)


def test_vit_s_bf16_21_tiles():
    cfg, prm, X, lab = _inputs("small", n=21, bf16=True)
    _run(cfg, prm, X, lab, 1, BF16_TOL)


# ---- block-inputs-only activation policy (blocks are re-run inside the backward) ----------------
def test_tiny_fp32_recompute():
    cfg, prm, X, lab = _inputs("tiny")
    _run(cfg, prm, X, lab, 0, FP32_TOL, recompute=1)


def test_vit_s_bf16_21_tiles_recompute():
    cfg, prm, X, lab = _inputs("small", n=21, bf16=True)
    _run(cfg, prm, X, lab, 1, BF16_TOL, recompute=1)


@pytest.mark.parametrize("dtype", [0, 1])
def test_recompute_is_bit_identical_to_keeping_everything(dtype):
    # same kernels on the same inputs in the same order: re-running a block reproduces its activations exactly
    from slide_harness import GpuSlide
    cfg, prm, X, lab = _inputs("small", n=5, bf16=bool(dtype))
    cfg = replace(cfg, layers=3)
    prm = gen.make_params(cfg, 77, perturbed=True)
    outs = []
    for rc in (0, 1):
        print(f"case small/3 layers n=5 dtype={dtype} recompute={rc}", flush=True)
        g = GpuSlide(cfg, prm, dtype, X.shape[0], rc)
        outs.append(g.step(X, lab))
        if rc == 1:
            assert g.lib.slide_arena_bytes(5) < GpuSlide(cfg, prm, dtype, 5, 0).lib.slide_arena_bytes(5)
    a, b = outs
    assert a["loss"] == b["loss"]
    for k in ("H", "G", "alpha", "dX"):
        assert np.array_equal(a[k], b[k]), k
    for k in a["grads"]:
        assert np.array_equal(a["grads"][k], b["grads"][k]), k


# ---- the Small workload at its own size (256 ViT-S tiles) and a 336-tile slide -------------------------------
def _oracle_chunked(prm, X, label, cfg, chunk=16):
    """The oracle's whole-slide step with bounded memory: tile chunks, features first, each chunk's forward run
    again just before its backward (the result is the one-piece gradient: sums over chunks)."""
    import time
    from oracle import slide_oracle as so
    N = X.shape[0]
    t0 = time.time()
    ref = so.slide_step(prm, X.astype(np.float64), label, cfg,
                        chunks=[(lo, min(N, lo + chunk)) for lo in range(0, N, chunk)], keep_caches=False)
    print(f"oracle step over {N} tiles: {time.time() - t0:.0f} s", flush=True)
    return ref


@pytest.mark.timeout(900)
def test_small_256_tiles_fp32_and_bf16():
    """cfg 2: 256 tiles of 224 px through ViT-S/16, M_h 128, one logit; both precisions against one oracle run on
    inputs that lie on the bf16 grid (valid fp32 numbers as well)."""
    from oracle import slide_oracle as so
    from slide_harness import GpuSlide, compare_step
    cfg, prm, X, lab = _inputs("small", bf16=True)
    assert X.shape[0] == 256
    outs = {}
    for dtype in (0, 1):
        print(f"case small n=256 dtype={dtype} label={lab}", flush=True)
        g = GpuSlide(cfg, prm, dtype, X.shape[0])
        outs[dtype] = g.step(X, lab)
        del g
    ref = _oracle_chunked(prm, X, lab, cfg)
    for dtype, tol in ((0, FP32_TOL), (1, BF16_TOL)):
        _, pool_same = so.pool_bwd(so.pool_fwd(prm, outs[dtype]["H"], lab, cfg)[4])
        errs, bad, kappa = compare_step(outs[dtype], ref, tol, cfg, None, pool_same)
        print(f"dtype={dtype} kappa={kappa:.1f} worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:8], flush=True)
        assert not bad, (dtype, bad)


@pytest.mark.timeout(600)
def test_vit_s_bf16_77_tiles_ragged_counts():
    """77 tiles of the medium workload: 15,169 token rows (59 whole 256-row tiles and 65 rows: the large-M forward and
    input-gradient kernels with a ragged last tile, the periodic position table of the patch embedding crossing tile
    boundaries at every phase) and a tile count that is no multiple of the 16 rows a lane group of the position-gradient
    sum takes at a time."""
    from slide_harness import GpuSlide, compare_step
    from oracle import slide_oracle as so
    cfg, _ = gen.CONFIGS["medium"]
    ds, ws, ls = gen.SEEDS["medium"]
    n = 77
    prm = {k: gen.to_bf16_grid(v) for k, v in gen.make_params(cfg, ws, perturbed=True).items()}
    X = gen.to_bf16_grid(gen.make_pixels(cfg, n, ds, first_tile=1024))
    lab = gen.make_label(cfg, ls)
    print(f"case medium tiles 1024..1100 n={n} dtype=1 label={lab}", flush=True)
    g = GpuSlide(cfg, prm, 1, n)
    out = g.step(X, lab)
    ref = _oracle_chunked(prm, X, lab, cfg)
    _, pool_same = so.pool_bwd(so.pool_fwd(prm, out["H"], lab, cfg)[4])
    errs, bad, kappa = compare_step(out, ref, BF16_TOL, cfg, None, pool_same)
    print(f"kappa={kappa:.1f} worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:8], flush=True)
    assert not bad, bad


@pytest.mark.timeout(900)
def test_vit_s_bf16_336_tiles_large_m_kernels_and_determinism():
    """336 consecutive tiles of the medium workload as a slide of their own: 66,192 token rows, so every
    activation-side GEMM runs several output tiles per workgroup of the large-M kernel (its background epilogue, in
    the forward and in both input-gradient epilogues) and every weight gradient runs the large-M kernel with the
    fused bias sums.  (a) whole step against the oracle; (b) encoder backward seeded with the ORACLE's feature
    gradients against the oracle's encoder gradients; (c) the same step twice gives the same bits."""
    import torch
    from slide_harness import GpuSlide, compare_step, rel_l2
    from oracle import slide_oracle as so
    cfg, _ = gen.CONFIGS["medium"]
    ds, ws, ls = gen.SEEDS["medium"]
    n = 336
    prm = {k: gen.to_bf16_grid(v) for k, v in gen.make_params(cfg, ws, perturbed=True).items()}
    X = gen.to_bf16_grid(gen.make_pixels(cfg, n, ds, first_tile=512))
    lab = gen.make_label(cfg, ls)
    print(f"case medium tiles 512..847 n={n} dtype=1 label={lab}", flush=True)
    g = GpuSlide(cfg, prm, 1, n)
    out = g.step(X, lab)
    again = g.step(X, lab)
    assert out["loss"] == again["loss"]
    for k in ("H", "G", "alpha", "dX", "logits"):
        assert np.array_equal(out[k], again[k]), k
    for k in out["grads"]:
        assert np.array_equal(out["grads"][k], again["grads"][k]), k
    print("two runs bit-identical", flush=True)
    ref = _oracle_chunked(prm, X, lab, cfg)
    _, pool_same = so.pool_bwd(so.pool_fwd(prm, out["H"], lab, cfg)[4])
    errs, bad, kappa = compare_step(out, ref, BF16_TOL, cfg, None, pool_same)
    print(f"kappa={kappa:.1f} worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:8], flush=True)
    assert not bad, bad
    # (b) encoder backward alone, seeded with the oracle's G
    px = g.to_dev(X)
    feats = torch.zeros((n, cfg.dim), device=g.dev)
    dpx = torch.zeros_like(px)
    g.lib.encoder_fwd_tiles(px, n, feats, 1)
    Gs = torch.from_numpy(ref["G"].astype(np.float32)).to(g.dev)
    g.lib.encoder_bwd_tiles(Gs, n, 0, dpx)
    torch.cuda.synchronize()
    gc = g.grads_dict()
    D = cfg.dim
    e3 = {"dX": rel_l2(dpx.float().cpu().numpy(), ref["dX"])}
    for k, v in ref["grads"].items():
        if k.startswith(("mil.", "head.")):
            continue
        a = gc[k]
        if k.endswith("qkv.b"):
            e3[k + "[q,v]"] = rel_l2(np.concatenate([a[:D], a[2 * D:]]), np.concatenate([v[:D], v[2 * D:]]))
            e3[k + "[k]abs"] = float(np.linalg.norm(a[D:2 * D]) / np.linalg.norm(v))
        else:
            e3[k] = rel_l2(a, v)
    print("encoder backward seeded with the oracle's G:", sorted(e3.items(), key=lambda kv: -kv[1])[:6], flush=True)
    assert all(v <= BF16_TOL for v in e3.values()), {k: v for k, v in e3.items() if v > BF16_TOL}
