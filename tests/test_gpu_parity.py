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
