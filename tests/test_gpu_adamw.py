"""AdamW update through the C ABI (slide_adamw_step) vs the CPU oracle (needs an MI355X).

Tolerances: the kernel works in fp32 on fp32 state.  Parameters, m and v carry half an ulp (6e-8 relative) per step:
relative L2 <= 1e-6 after three steps.  The applied change theta_t - theta_0 is of size lr against parameters of size
0.02, so the rounding of theta shows in it as 6e-8 * 0.02 / lr ~ 2e-5 relative at lr = 5e-5: <= 1e-4 there, scaled
with 1 / lr below that learning rate."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


def _lib():
    from paper_2403_04865_amd import SlideLib
    from slide_harness import lib_config
    cfg, _ = gen.CONFIGS["tiny"]
    return SlideLib(lib_config(cfg, 0))


def _run_case(n, steps, lr, wd, offset=0, seed=11):
    import torch
    from oracle.adamw_oracle import adamw_step
    from slide_harness import rel_l2
    print(f"case adamw n={n} steps={steps} lr={lr} wd={wd} offset={offset}", flush=True)
    lib = _lib()
    rng = np.random.Generator(np.random.PCG64(seed))
    th0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    # gradients over many decades, some exactly zero (parameters a slide did not touch)
    gs = [(rng.standard_normal(n) * 10.0 ** rng.integers(-7, 1, size=n) * (rng.random(n) > 0.05)).astype(np.float32)
          for _ in range(steps)]
    dev = torch.device("cuda:0")

    def dbuf(a):   # device copy starting `offset` floats into an allocation (offset != 0: not 16-byte aligned)
        t = torch.zeros(n + offset + 4, dtype=torch.float32, device=dev)
        t[offset:offset + n] = torch.from_numpy(a)
        return t, t[offset:offset + n]

    Pfull, P = dbuf(th0)
    Mfull, M = dbuf(np.zeros(n, np.float32))
    Vfull, V = dbuf(np.zeros(n, np.float32))
    th, m, v = th0.astype(np.float64), np.zeros(n), np.zeros(n)
    # the ABI takes the hyper-parameters as float: both sides use those float values (1 - beta2 of the float nearest
    # to 0.999 differs from 0.001 by 1.3e-5 relative)
    lr, wd, b1, b2, eps = (float(np.float32(x)) for x in (lr, wd, 0.9, 0.999, 1e-8))
    for t in range(1, steps + 1):
        Gfull, G = dbuf(gs[t - 1])
        lib.slide_adamw_step(P, G, M, V, n, t, lr, b1, b2, eps, wd)
        torch.cuda.synchronize()
        th, m, v = adamw_step(th, gs[t - 1].astype(np.float64), m, v, t, lr, b1, b2, eps, wd)
    p, mm, vv = P.cpu().numpy().astype(np.float64), M.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64)
    errs = {"theta": rel_l2(p, th), "m": rel_l2(mm, m), "v": rel_l2(vv, v), "delta": rel_l2(p - th0, th - th0)}
    print(errs, flush=True)
    delta_tol = 1e-4 * max(1.0, 5e-5 / lr)
    assert errs["theta"] <= 1e-6 and errs["m"] <= 1e-6 and errs["v"] <= 1e-6 and errs["delta"] <= delta_tol, errs
    # nothing outside the n elements was written
    for full in (Pfull, Mfull, Vfull):
        assert not full[:offset].any() and not full[offset + n:].any()


def test_adamw_vit_s_parameter_count():      # every parameter of the ViT-S workload, the paper's peak learning rate
    cfg, _ = gen.CONFIGS["large"]
    from paper_2403_04865_amd import SlideLib
    from slide_harness import lib_config
    n = SlideLib(lib_config(cfg, 1)).slide_param_count()
    _run_case(n, 3, 5e-5, 0.01)


def test_adamw_ragged_count():               # count that is no multiple of 4: vector body + scalar tail
    _run_case(100003, 3, 1e-4, 0.01)


def test_adamw_unaligned_buffers():          # buffers that are not 16-byte aligned take the scalar kernel
    _run_case(4099, 2, 1e-4, 0.0, offset=1)


def test_adamw_tiny_and_no_decay():
    _run_case(1, 4, 1e-6, 0.0)


def test_adamw_rejects_bad_arguments():
    import torch
    lib = _lib()
    dev = torch.device("cuda:0")
    a = torch.zeros(8, device=dev)
    for kw in (dict(count=0), dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(lr=-1.0), dict(eps=-1.0),
               dict(weight_decay=-0.5)):
        args = dict(count=8, step=1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
        args.update(kw)
        with pytest.raises(Exception):
            lib.slide_adamw_step(a, a, a, a, **args)
    with pytest.raises(Exception):
        lib.slide_adamw_step(None, a, a, a, 8, 1, 1e-3)
