"""slide_step_chunked (a slide that goes through the encoder in chunks, for arenas smaller than the slide) through the
C ABI: against the CPU oracle's whole-slide step, and against the library's own whole-slide step (needs an MI355X).

The paper's equivalence claim (Results, gradient equivalence) is what makes the chunked step exact: once the feature
gradients of the whole slide are known, the parameter gradients are a sum over any partition of the tiles."""
import numpy as np
import pytest

import gen
from test_gpu_parity import BF16_TOL, FP32_TOL, _inputs

pytestmark = pytest.mark.gpu


def _chunked(cfg, prm, X, dtype, chunk, recompute=0):
    from slide_harness import GpuSlide
    N = X.shape[0]
    return GpuSlide(cfg, prm, dtype, N, recompute, arena_bytes=lambda lib: lib.slide_chunked_arena_bytes(N, chunk))


@pytest.mark.parametrize("chunk", [5, 13, 1])
def test_chunked_tiny_fp32_vs_oracle(chunk):   # 13 tiles in chunks of 5 (ragged last chunk), one chunk, single tiles
    from oracle import slide_oracle as so
    from slide_harness import compare_step
    cfg, prm, X, lab = _inputs("tiny", n=13, std=0.05)
    print(f"case chunked tiny fp32 n=13 chunk={chunk}", flush=True)
    g = _chunked(cfg, prm, X, 0, chunk)
    out = g.step_chunked(X, lab, chunk)
    ref = so.slide_step(prm, X.astype(np.float64), lab, cfg)
    _, pool_same = so.pool_bwd(so.pool_fwd(prm, out["H"], lab, cfg)[4])
    errs, bad, kappa = compare_step(out, ref, FP32_TOL, cfg, None, pool_same)
    print("worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:6], flush=True)
    assert not bad, bad


@pytest.mark.parametrize("recompute", [0, 1])
def test_chunked_vit_s_bf16_vs_oracle(recompute):   # ViT-S blocks, 21 tiles in chunks of 8 (8 + 8 + 5), bf16 path
    from oracle import slide_oracle as so
    from slide_harness import GATE, GpuSlide, compare_step, feature_spread, rel_l2
    cfg, prm, X, lab = _inputs("small", n=21, bf16=True)
    print(f"case chunked small bf16 n=21 chunk=8 recompute={recompute}", flush=True)
    g = _chunked(cfg, prm, X, 1, 8, recompute)
    assert g.lib.slide_chunked_arena_bytes(21, 8) < g.lib.slide_arena_bytes(21)
    out = g.step_chunked(X, lab, 8)
    ref = so.slide_step(prm, X.astype(np.float64), lab, cfg)
    _, pool_same = so.pool_bwd(so.pool_fwd(prm, out["H"], lab, cfg)[4])
    errs, bad, kappa = compare_step(out, ref, BF16_TOL, cfg, None, pool_same)
    print(f"kappa={kappa:.1f} worst:", sorted(errs.items(), key=lambda kv: -kv[1])[:6], flush=True)
    assert not bad, bad
    # against the library's one-piece step: both lie within the tolerance of the oracle, so within twice the tolerance
    # of each other (the row count of a call selects the GEMM kernel, so the bf16 roundings differ); the aggregator's
    # gate tensors see the features only through differences between rows, which amplifies that by kappa
    whole = GpuSlide(cfg, prm, 1, 21, recompute).step(X, lab)
    d = {k: rel_l2(out[k], whole[k]) for k in ("logits", "alpha", "H", "G", "dX")}
    d.update({k: rel_l2(out["grads"][k], v) for k, v in whole["grads"].items() if np.linalg.norm(v) > 0})
    kap = max(1.0, feature_spread(whole["H"]))
    badw = {k: v for k, v in d.items() if not v <= 2 * BF16_TOL * (kap if k in GATE else 1.0)}
    assert not badw, badw
    # accumulate: a second chunked step on top doubles every gradient
    out2 = g.step_chunked(X, lab, 8, accumulate=True)
    for k, v in out["grads"].items():
        if np.linalg.norm(v) > 0:
            assert rel_l2(out2["grads"][k], 2.0 * v) <= 1e-5, k


def test_chunked_rejects_small_arena_and_bad_arguments():
    import torch
    from paper_2403_04865_amd.binding import SlideError
    from slide_harness import GpuSlide
    cfg, prm, X, lab = _inputs("tiny", n=13)
    g = GpuSlide(cfg, prm, 0, 13, arena_bytes=lambda lib: lib.slide_chunked_arena_bytes(13, 4))
    px = g.to_dev(X)
    loss = torch.zeros(1, device=g.dev)
    with pytest.raises(SlideError) as e:
        g.lib.slide_step_chunked(px, 13, 8, lab, 0, loss)      # chunks of 8 need more than the arena for chunks of 4
    assert e.value.code == -2
    with pytest.raises(SlideError) as e:
        g.lib.slide_step_chunked(px, 13, 0, lab, 0, loss)
    assert e.value.code == -1
    with pytest.raises(SlideError) as e:
        g.lib.slide_step_chunked(px, 13, 4, 7, 0, loss)        # label out of range
    assert e.value.code == -1
    g.lib.slide_step_chunked(px, 13, 4, lab, 0, loss)           # and the fitting call works
    torch.cuda.synchronize()
    assert np.isfinite(loss.item())
