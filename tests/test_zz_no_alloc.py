"""mil_pool_fwd_static (work space inside the library's device code, no allocation) against mil_pool_fwd on the same
inputs, through the C ABI (needs an MI355X): two calls in a row, the second over fewer rows."""
from dataclasses import replace

import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,dtype,rows", [("large", 1, (8192, 1000)), ("medium", 1, (40000 + 13, 4096 + 77)),
                                             ("full", 1, (4096 + 5, 700)), ("tiny", 0, (300, 16))])
def test_static_pool_forward_matches_arena_pool_forward(name, dtype, rows):
    import torch
    from paper_2403_04865_amd import SlideLib, SlideError, config_from
    cfg, _ = gen.CONFIGS[name]
    _, ws, ls = gen.SEEDS[name]
    dev = torch.device("cuda:0")
    prm = gen.make_params(cfg, ws, perturbed=True)
    for k in ("mil.V.W", "mil.U.W", "mil.w"):
        prm[k] = prm[k] * 4.0
    lib = SlideLib(config_from(cfg, dtype))
    flat = np.zeros(lib.slide_param_count(), dtype=np.float32)
    for nm, off, ln in lib.param_layout():
        flat[off:off + ln] = np.asarray(prm[nm], dtype=np.float32).reshape(-1)
    params = torch.from_numpy(flat).to(dev)
    grads = torch.zeros_like(params)
    lab = gen.make_label(cfg, ls)
    free = SlideLib(config_from(cfg, dtype))      # never bound: the static entry point needs the shapes only
    for N in rows:
        print(f"case static pool {name} dtype={dtype} N={N}", flush=True)
        H = torch.from_numpy(gen.make_features(cfg, N, 11)).to(dev)
        nbytes = lib.slide_pool_arena_bytes(N)
        arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        o = (-arena.data_ptr()) % 256
        lib.slide_bind(params, grads, arena[o:o + nbytes])
        out = {}
        for which in ("arena", "static"):
            loss = torch.full((1,), -1.0, device=dev)
            logits = torch.full((cfg.n_classes,), -1.0, device=dev)
            alpha = torch.full((N,), -1.0, device=dev)
            if which == "arena":
                lib.mil_pool_fwd(H, N, lab, loss, logits, alpha)
            else:
                free.mil_pool_fwd_static(params, H, N, lab, loss, logits, alpha)
            torch.cuda.synchronize()
            out[which] = (loss.cpu().numpy(), logits.cpu().numpy(), alpha.cpu().numpy())
        for a, b, what in zip(out["arena"], out["static"], ("loss", "logits", "alpha")):
            assert np.isfinite(b).all(), what
            assert np.array_equal(a, b), (what, N)          # same kernels on the same inputs: the same bits
        assert abs(float(out["static"][2].sum()) - 1.0) < 1e-4
    # beyond the documented maximum: refused, nothing launched
    with pytest.raises(SlideError) as e:
        free.mil_pool_fwd_static(params, H, 65536 + 1, lab, None, None, None)
    assert e.value.code == -2
