"""Gated-attention MIL pool through the C ABI (mil_pool_fwd / mil_pool_bwd) vs the CPU oracle on the same
feature matrix, at the real shapes of the workloads (needs an MI355X)."""
from dataclasses import replace

import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4
BF16_TOL = 2e-2


def _pool_case(name, N, dtype, seed=5, mil_hidden=None, n_classes=None, label=None, w_scale=1.0):
    import torch
    from oracle import slide_oracle as so
    from paper_2403_04865_amd import SlideLib
    from slide_harness import lib_config, rel_l2
    cfg, _ = gen.CONFIGS[name]
    if mil_hidden:
        cfg = replace(cfg, mil_hidden=mil_hidden)
    if n_classes:
        cfg = replace(cfg, n_classes=n_classes)
    _, ws, ls = gen.SEEDS[name]
    print(f"case pool {name} N={N} D={cfg.dim} Mh={cfg.mil_hidden} C={cfg.n_classes} dtype={dtype}", flush=True)
    prm = gen.make_params(cfg, ws, perturbed=True)
    if dtype == 1:
        prm = {k: gen.to_bf16_grid(v) for k, v in prm.items()}
    # the pool reads only the aggregator tensors; a larger init makes the gates leave their linear range
    for k in ("mil.V.W", "mil.U.W", "mil.w"):
        prm[k] = (prm[k] * 4.0).astype(np.float64)
    prm["mil.w"] = prm["mil.w"] * w_scale
    print("sum |w| =", float(np.abs(prm["mil.w"]).sum()), flush=True)
    if dtype == 1:
        prm = {k: gen.to_bf16_grid(v) for k, v in prm.items()}
    Hf = gen.make_features(cfg, N, seed)
    lab = gen.make_label(cfg, ls) if label is None else label
    dev = torch.device("cuda:0")
    lib = SlideLib(lib_config(cfg, dtype))
    layout = lib.param_layout()
    flat = np.zeros(lib.slide_param_count(), dtype=np.float32)
    for nm, off, ln in layout:
        flat[off:off + ln] = np.asarray(prm[nm], dtype=np.float32).reshape(-1)
    params = torch.from_numpy(flat).to(dev)
    grads = torch.zeros_like(params)
    nbytes = lib.slide_pool_arena_bytes(N)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    o = (-arena.data_ptr()) % 256
    arena = arena[o:o + nbytes]
    lib.slide_bind(params, grads, arena)
    H = torch.from_numpy(Hf).to(dev)
    loss = torch.zeros(1, device=dev)
    logits = torch.zeros(cfg.n_classes, device=dev)
    alpha = torch.zeros(N, device=dev)
    G = torch.zeros_like(H)
    lib.mil_pool_fwd(H, N, lab, loss, logits, alpha)
    lib.mil_pool_bwd(H, N, lab, G, 0)
    torch.cuda.synchronize()
    rl, ry, ra, rz, cache = so.pool_fwd(prm, Hf.astype(np.float64), lab, cfg)
    rG, rg = so.pool_bwd(cache)
    g = grads.cpu().numpy().astype(np.float64)
    errs = {"loss": abs(loss.item() - rl) / max(abs(rl), 1e-12), "logits": rel_l2(logits.cpu().numpy(), ry),
            "alpha": rel_l2(alpha.cpu().numpy(), ra), "G": rel_l2(G.cpu().numpy(), rG)}
    for nm, off, ln in layout:
        if nm.startswith(("mil.", "head.")):
            errs[nm] = rel_l2(g[off:off + ln], rg[nm].reshape(-1))
    tol = FP32_TOL if dtype == 0 else BF16_TOL
    print("worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:6], flush=True)
    assert abs(alpha.sum().item() - 1.0) < 1e-4
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad


# matrix-core forward (bf16 path), every (D, M_h) that is built, real row counts
def test_pool_bf16_large_shape():          # 8192 x 384, M_h 256, 4 classes
    _pool_case("large", 8192, 1)


def test_pool_bf16_medium_shape():         # 2048 x 384, M_h 128, one logit
    _pool_case("medium", 2048, 1)


def test_pool_bf16_ragged_rows():          # row count that is no multiple of the 64-row block, single class
    _pool_case("medium", 1000 + 37, 1, label=1)


def test_pool_bf16_many_rows():            # 16-17 blocks per workgroup of the persistent forward (its register roles
    _pool_case("medium", 131072 + 4096 + 19, 1, label=1)   # repeat every 6), unevenly; large-M weight-gradient GEMM; ragged tail


def test_pool_bf16_mh256_many_rows():       # M_h = 256 above 32768 rows: forward in two passes of 128 gate units each
    _pool_case("large", 32768 + 4096 + 7, 1)   # (the backward takes M_h = 256 as two halves at every size)


def test_pool_bf16_large_logit_weights():  # sum |w| > 40: the logit bound is no usable softmax shift, running maximum instead
    _pool_case("medium", 4096 + 77, 1, w_scale=30.0)


def test_pool_bf16_vit_b_shape():          # 768-wide features (32-row blocks), M_h 256
    _pool_case("full", 4096 + 5, 1)


def test_pool_bf16_vit_b_mh128():
    _pool_case("full", 1024, 1, mil_hidden=128, n_classes=3, label=2)


# plain-ALU kernels: fp32 path at the same shapes, and small bags on the bf16 path
def test_pool_fp32_large_shape():
    _pool_case("large", 8192, 0)


def test_pool_fp32_ragged_rows():
    _pool_case("medium", 1000 + 37, 0)


def test_pool_bf16_small_bag():            # fewer rows than the matrix-core kernel takes
    _pool_case("medium", 100, 1)


def test_pool_single_row():                # N = 1: alpha = 1, z = h_1
    _pool_case("medium", 1, 0)


def test_pool_over_more_rows_invalidates_a_saved_step():
    """A pool call over more rows than the saved slide step has tiles lays its work space over that step's features:
    the step must be dropped (slide_step_bwd reports SLIDE_ESTATE) instead of running on overwritten rows.  A pool
    call over no more rows than the step leaves it intact."""
    import torch
    from paper_2403_04865_amd import SlideError
    from slide_harness import GpuSlide
    cfg, n = gen.CONFIGS["tiny"]
    ds, ws, ls = gen.SEEDS["tiny"]
    prm = gen.make_params(cfg, ws, perturbed=True)
    X = gen.make_pixels(cfg, n, ds, kind="uniform")
    print("case pool call between slide_step_fwd and slide_step_bwd (tiny, fp32)", flush=True)
    g = GpuSlide(cfg, prm, 0, 64)      # arena sized for 64 tiles: a 48-row pool fits beside a 16-tile step
    dev = g.dev
    ref = g.step(X, 1)
    px = g.to_dev(X)
    loss = torch.zeros(1, device=dev)
    feats = torch.from_numpy(gen.make_features(cfg, 48, 3)).to(dev)
    # same number of rows: the step survives and gives the same gradients
    g.lib.slide_step_fwd(px, n, 1, loss, None, None)
    g.lib.mil_pool_fwd(feats[:n].contiguous(), n, 1, loss, None, None)
    g.lib.slide_step_bwd(0, None)
    torch.cuda.synchronize()
    same = g.grads_dict()
    for k in ref["grads"]:
        assert np.array_equal(ref["grads"][k], same[k]), k
    # more rows: the step is gone
    g.lib.slide_step_fwd(px, n, 1, loss, None, None)
    g.lib.mil_pool_fwd(feats, 48, 1, loss, None, None)
    with pytest.raises(SlideError) as e:
        g.lib.slide_step_bwd(0, None)
    assert e.value.code == -4
    torch.cuda.synchronize()
