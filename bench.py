#!/usr/bin/env python3
"""Benchmark of the slide step on one MI355X.

A "step" is one whole slide step (slide_step_fwd + slide_step_bwd: encoder forward and backward
over every tile, gated-attention pool forward and backward, all parameter gradients) on one
synthetic slide that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|medium|small|full]
    python bench.py --workload rn18|rn50      the same step with a ResNet tile encoder (include/resnet.h)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# model FLOPs per tile, forward + backward (2mnk per GEMM, both attention GEMMs, dgrad + wgrad,
# no pixel gradient)
def model_flops_per_tile(cfg):
    T, D, F, H = cfg.tokens, cfg.dim, cfg.ffn, cfg.heads
    dh = D // H
    g2 = T - 1
    per_layer = 2 * T * D * 3 * D + 2 * T * D * D + 2 * 2 * T * D * F + 2 * 2 * H * T * T * dh
    fwd = 2 * g2 * cfg.patch_dim * D + cfg.layers * per_layer
    bwd = 2 * g2 * cfg.patch_dim * D + 2 * cfg.layers * per_layer   # patch embed: wgrad only
    return fwd + bwd


# what the exact pruning of the last block leaves out (its output is read at the CLS row only: projection and MLP on
# one row instead of T, attention for one query instead of T), forward + backward
def pruned_flops_per_tile(cfg):
    T, D, F, H = cfg.tokens, cfg.dim, cfg.ffn, cfg.heads
    dh = D // H
    rows = (T - 1) * (2 * D * D + 2 * 2 * D * F) + 2 * 2 * H * (T - 1) * T * dh
    return 3 * rows


PEAK = {"mfma_bf16": 2.5e15, "hbm": 8e12}


def pool_sweep(a):
    """Achieved HBM bandwidth of the pool kernels alone (mil_pool_fwd / mil_pool_bwd through the C ABI) over feature
    matrices far larger than the caches: N = 2^13 .. 2^22 rows of 384 floats, M_h = 128, one logit.  Algorithmic
    bytes: forward N*D*4 (every feature row read once), backward 2*N*D*4 (rows read once, gradient rows written
    once).  Times are HIP events around the kernels of each call, on the launch stream, over --pool-reps calls after
    --pool-warmup untimed ones.  The forward is timed twice: in a run of forward calls (fwd_*), where the same launch
    keeps getting faster for more than 70 ms (power management), and as the first stage of the backward call
    (fwd_in_bwd_*), between other kernels."""
    import numpy as np
    import torch
    import gen
    from dataclasses import replace
    from paper_2403_04865_amd import config_from as lib_config
    from paper_2403_04865_amd import SlideLib
    cfg, _ = gen.CONFIGS["medium"]
    cfg = replace(cfg, mil_hidden=a.pool_hidden)
    dev = torch.device("cuda:0")
    lib = SlideLib(lib_config(cfg, 1))
    prm = gen.make_params(cfg, gen.SEEDS["medium"][1])
    flat = np.zeros(lib.slide_param_count(), dtype=np.float32)
    for name, off, ln in lib.param_layout():
        flat[off:off + ln] = prm[name].reshape(-1)
    params = torch.from_numpy(flat).to(dev)
    grads = torch.zeros_like(params)
    names = lib.kernel_names()
    rows = []
    for lg in range(a.pool_min_log2, a.pool_max_log2 + 1):
        N = 1 << lg
        nbytes = lib.slide_pool_arena_bytes(N)
        arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        o = (-arena.data_ptr()) % 256
        lib.slide_bind(params, grads, arena[o:o + nbytes])
        H = torch.from_numpy(gen.make_features(cfg, min(N, 1 << 16), 9)).to(dev)
        if N > H.shape[0]:
            H = H.repeat(N // H.shape[0], 1).contiguous()
        G = torch.empty_like(H)
        loss = torch.zeros(1, device=dev)
        res = {"N": N, "feature_MB": round(N * cfg.dim * 4 / 1e6, 1)}
        # fwd_in_bwd: the forward kernels as they run inside the backward call (which recomputes the forward first),
        # i.e. between other kernels instead of back to back with themselves
        for which, kid in (("fwd", names.index("pool_fwd")), ("bwd", names.index("pool_bwd")),
                           ("fwd_in_bwd", names.index("pool_fwd"))):
            reps, warm = a.pool_reps, a.pool_warmup
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for it in range(warm + reps):
                if it == warm:
                    torch.cuda.synchronize()
                    lib.slide_prof_begin(kid)
                    e0.record()
                if which == "fwd":
                    lib.mil_pool_fwd(H, N, 1, loss, None, None)
                else:
                    lib.mil_pool_bwd(H, N, 1, G, 0)
            e1.record()
            torch.cuda.synchronize()
            ms, n, _, by = lib.slide_prof_end()
            ms /= max(n, 1)
            # the whole ABI call (backward: forward recomputation + row kernel + weight-gradient reductions)
            if which != "fwd_in_bwd":
                res[which + "_call_us"] = round(e0.elapsed_time(e1) / reps * 1e3, 1)
            alg = N * cfg.dim * 4 * (2 if which == "bwd" else 1)
            res[which + "_us"] = round(ms * 1e3, 1)
            res[which + "_GBps"] = round(alg / (ms * 1e-3) / 1e9, 1)
            res[which + "_frac_hbm"] = round(alg / (ms * 1e-3) / PEAK["hbm"], 4)
            # the same time against half the bytes: what the fraction would be if the features were counted as bf16
            res[which + "_frac_hbm_if_bf16_features"] = round(0.5 * alg / (ms * 1e-3) / PEAK["hbm"], 4)
        rows.append(res)
        print(json.dumps(res), flush=True)
        del arena, H, G
        torch.cuda.empty_cache()
    print(json.dumps({"pool_sweep": rows, "D": cfg.dim, "mil_hidden": cfg.mil_hidden, "peak_GBps": PEAK["hbm"] / 1e9,
                      "bytes_basis": "features and feature gradients are float32: forward N*D*4, backward 2*N*D*4 bytes"}))


def adamw_bench(a):
    """AdamW update of every parameter of the workload's model: achieved HBM bandwidth against the 28 bytes per
    parameter the update has to move (read theta, g, m, v; write theta, m, v), HIP events on the launch stream."""
    import numpy as np
    import torch
    import gen
    from paper_2403_04865_amd import config_from as lib_config
    from paper_2403_04865_amd import SlideLib
    cfg, _ = gen.CONFIGS[a.workload]
    lib = SlideLib(lib_config(cfg, 1))
    n = lib.slide_param_count()
    dev = torch.device("cuda:0")
    rng = np.random.Generator(np.random.PCG64(7))
    P = torch.from_numpy((rng.standard_normal(n) * 0.02).astype(np.float32)).to(dev)
    G = torch.from_numpy((rng.standard_normal(n) * 1e-3).astype(np.float32)).to(dev)
    M = torch.zeros_like(P)
    V = torch.zeros_like(P)
    for t in range(1, a.warmup + 1):
        lib.slide_adamw_step(P, G, M, V, n, t, 5e-5)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(a.warmup + 1, a.warmup + a.steps + 1):
        lib.slide_adamw_step(P, G, M, V, n, t, 5e-5)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    gbps = n * 28 / (ms * 1e-3) / 1e9
    print(json.dumps({"adamw": {"workload": a.workload, "parameters": n, "us_per_update": round(ms * 1e3, 1),
                                "bytes_per_parameter": 28, "achieved_GBps": round(gbps, 1), "peak_GBps": PEAK["hbm"] / 1e9,
                                "frac": round(gbps * 1e9 / PEAK["hbm"], 4), "steps": a.steps, "warmup": a.warmup}}))


def calib_copy(a):
    """One warm-up and three launches of the library's plain copy kernel over --calib-copy bytes: the known-size
    kernel whose FETCH_SIZE / WRITE_SIZE readings give the scale of those counters."""
    import torch
    from paper_2403_04865_amd import SlideLib, SlideConfig
    lib = SlideLib(SlideConfig(32, 8, 64, 2, 2, 4, 32, 1))
    n = a.calib_copy // 16 * 16
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    for _ in range(4):
        lib.slide_calib_copy(dst, src, n)
    torch.cuda.synchronize()
    assert bool((dst[:4096] == 1).all())
    print(json.dumps({"calib_copy_bytes": n, "launches": 4}))


def resnet_model_flops_per_tile(cfg):
    """Model FLOPs of one tile through the ResNet encoder, forward + backward: 2 * positions * Cout * Cin * k * k per
    convolution; backward = input gradient + weight gradient of every convolution except the stem's input gradient."""
    import gen
    S = cfg.tile
    fwd = 2.0 * (S // 2) ** 2 * cfg.width * 3 * 49
    bwd = fwd
    H = S // 4
    for b in gen.resnet_blocks(cfg):
        Ho = H // b["stride"]
        if cfg.block == "basic":
            convs = [(Ho, b["mid"], b["cin"], 3), (Ho, b["cout"], b["mid"], 3)]
        else:
            convs = [(H, b["mid"], b["cin"], 1), (Ho, b["mid"], b["mid"], 3), (Ho, b["cout"], b["mid"], 1)]
        if b["down"]:
            convs.append((Ho, b["cout"], b["cin"], 1))
        f = sum(2.0 * h * h * co * ci * k * k for h, co, ci, k in convs)
        fwd += f
        bwd += 2 * f
        H = Ho
    return fwd + bwd


def resnet_bench(a):
    """The slide step with a ResNet tile encoder (resnet_slide_step_fwd + resnet_slide_step_bwd) on one synthetic slide
    resident in HBM; same output contract as the default run."""
    import numpy as np
    import torch
    import gen
    from paper_2403_04865_amd import ResNetLib, resnet_config_from
    cfg, N = gen.RESNET_CONFIGS[a.workload]
    if a.tiles:
        N = a.tiles
    ds, ws, ls = gen.RESNET_SEEDS[a.workload]
    dev = torch.device("cuda:0")
    lib = ResNetLib(resnet_config_from(cfg))
    prm = gen.make_resnet_params(cfg, ws)
    flat = np.zeros(lib.resnet_param_count(), dtype=np.float32)
    for name, off, ln in lib.param_layout():
        flat[off:off + ln] = prm[name].reshape(-1)
    params = torch.from_numpy(flat).to(dev)
    grads = torch.zeros_like(params)
    nbytes = lib.resnet_arena_bytes(N)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    o = (-arena.data_ptr()) % 256
    arena = arena[o:o + nbytes]
    lib.resnet_bind(params, grads, arena)
    t0 = time.time()
    px = torch.empty((N, 3, cfg.tile, cfg.tile), dtype=torch.bfloat16, device=dev)
    workers = min(16, os.cpu_count() or 1)
    for lo in range(0, N, 512):
        hi = min(N, lo + 512)
        px[lo:hi] = torch.from_numpy(gen.make_pixels(cfg, hi - lo, ds, first_tile=lo, workers=workers)).to(dev).to(torch.bfloat16)
    rng = np.random.Generator(np.random.PCG64(ls))
    label = int(rng.random() < 0.5) if cfg.n_classes == 1 else int(rng.integers(0, cfg.n_classes))
    gen_s = time.time() - t0
    loss = torch.zeros(1, device=dev)
    logits = torch.zeros(cfg.n_classes, device=dev)
    stream = torch.cuda.current_stream()

    def one_step():
        lib.resnet_slide_step_fwd(px, N, label, loss, logits, None, stream)
        lib.resnet_slide_step_bwd(0, stream)

    for _ in range(a.warmup):
        one_step()
    torch.cuda.synchronize()
    names = lib.kernel_names()
    prof = a.prof_kernel if a.prof_kernel in names else "conv_fwd"
    lib.resnet_prof_begin(names.index(prof))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k_ms, k_n, k_flops, k_bytes = lib.resnet_prof_end()
    peak_alloc = torch.cuda.max_memory_allocated() / 1e9
    stored = load_traffic(a.workload) if not a.tiles else None
    roof = roofline_of(prof, k_ms, k_n, k_flops, k_bytes, dt * 1e3,
                       (stored or {}).get("conv_nt" if prof in ("conv_fwd", "conv_dgrad") else prof))
    lib.resnet_prof_begin(-1)
    t1 = time.perf_counter()
    one_step()
    torch.cuda.synchronize()
    all_ms = (time.perf_counter() - t1) * 1e3
    lib.resnet_prof_end()
    roof_all = []
    for i, nm in enumerate(names):
        f_ms, f_n, f_fl, f_by = lib.resnet_prof_family(i)
        if f_n:
            # forward and input gradient are launches of one kernel: the counters know them as one family
            key = "conv_nt" if nm in ("conv_fwd", "conv_dgrad") else nm
            roof_all.append(roofline_of(nm, f_ms, f_n, f_fl, f_by, all_ms, (stored or {}).get(key)))
    roof_all.sort(key=lambda r: -(r["share_of_step"] or 0))
    tiles_per_s = N * a.steps / dt
    mflops = resnet_model_flops_per_tile(cfg)
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import resnet_oracle as ro
        from threadpoolctl import threadpool_info
        nt = min(a.cpu_tiles, N)
        Xc = px[:nt].float().cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        ro.slide_step({k: v.astype(np.float64) for k, v in prm.items()}, Xc, label, cfg)
        cs = time.perf_counter() - t0
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        cpu = {"value": round(nt / cs, 3), "unit": "tiles/s", "cores": cores, "kind": "oracle",
               "sample": f"{nt} tiles of the same slide, fp64 numpy oracle, full fwd+bwd step"}
    out = {
        "metric": "tiles/sec fwd+bwd per slide step (1 MI355X); MFMA util % of bf16 peak",
        "value": round(tiles_per_s, 2), "unit": "tiles/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt / a.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {N} tiles {cfg.tile}x{cfg.tile}x3, ResNet {cfg.block} blocks {list(cfg.depths)} "
                               f"width {cfg.width}, batch statistics over all tiles, gated-attention MIL hidden "
                               f"{cfg.mil_hidden}, {cfg.n_classes} classes",
                   "tiles": N, "slide_steps_per_s": round(a.steps / dt, 4),
                   "model_gflop_per_tile": round(mflops / 1e9, 3),
                   "mfu_bf16_peak": round(tiles_per_s * mflops / PEAK["mfma_bf16"], 4),
                   "activation_policy": "all activations kept",
                   "arena_gb": round(nbytes / 1e9, 2), "peak_alloc_gb_of_288": round(peak_alloc, 2),
                   "loss": float(loss.item()), "input_gen_s": round(gen_s, 1)},
        "roofline": roof, "roofline_all": roof_all,
        "traffic_source": None if stored is None else {"kind": "stored", "file": f"profiles/traffic_{a.workload}.json",
                                                       "measured_at_commit": stored.get("_commit")},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def load_traffic(workload, kernel=None):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc (profiles/traffic_<workload>.json, written by
    `python -m paper_2403_04865_amd.pmc_traffic`; a STORED figure of an earlier run, not measured by this one: the
    file names the commit it was measured at); None when no measurement of this workload is stored.  Without
    `kernel`: the whole file."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        d = json.load(f)
    return d if kernel is None else d.get(kernel)


HBM_BOUND = ("ln_fwd", "ln_bwd", "pool_fwd", "pool_bwd", "colsum", "elementwise",
             "bn_stats", "bn_apply", "bn_bwd", "pooling", "mil_pool")


def roofline_of(name, ms, n, flops, nbytes, step_ms, traffic):
    """One family's figures from its HIP-event times: contractions against the dense bf16 MFMA peak, streaming kernels
    (algorithmic bytes) against the HBM peak."""
    hbm = name in HBM_BOUND
    if hbm:
        achieved = (nbytes / (ms * 1e-3)) / 1e9 if ms > 0 else 0.0
        peak, unit = PEAK["hbm"] / 1e9, "GB/s"
    else:
        achieved = (flops / (ms * 1e-3)) / 1e12 if ms > 0 else 0.0
        peak, unit = PEAK["mfma_bf16"] / 1e12, "TFLOP/s"
    return {"bound": "hbm" if hbm else "mfma", "kernel": name, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 4), "traffic": None if traffic is None else traffic["hbm_bytes_per_launch"],
            "algorithmic_bytes_per_launch": round(nbytes / max(n, 1)), "launches": n,
            "avg_launch_ms": round(ms / max(n, 1), 4), "share_of_step": round(ms / step_ms, 4) if step_ms > 0 else None}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--tiles", type=int, default=0, help="override the tile count")
    ap.add_argument("--chunk-tiles", type=int, default=0,
                    help="run the chunked step (slide_step_chunked) with this many tiles per encoder chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tiles", type=int, default=16)
    ap.add_argument("--prof-kernel", default="gemm_nt")
    ap.add_argument("--recompute", type=int, default=-1,
                    help="1 = keep block inputs only and re-run blocks in the backward (default: only for 'full')")
    ap.add_argument("--calib-copy", type=int, default=0, help="run the plain copy kernel over this many bytes and exit")
    ap.add_argument("--adamw", action="store_true", help="time the AdamW update of the workload's parameters instead")
    ap.add_argument("--pool-sweep", action="store_true", help="bandwidth sweep of the pool kernels instead of the step")
    ap.add_argument("--pool-hidden", type=int, default=128)
    ap.add_argument("--pool-min-log2", type=int, default=13)
    ap.add_argument("--pool-max-log2", type=int, default=22)
    ap.add_argument("--pool-reps", type=int, default=20, help="timed calls per size and direction")
    ap.add_argument("--pool-warmup", type=int, default=40,
                    help="untimed calls before them (the first ~40 ms of a run of these kernels are up to 40 % slower)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if a.pool_sweep:
        return pool_sweep(a)
    if a.adamw:
        return adamw_bench(a)
    if a.calib_copy:
        return calib_copy(a)

    import gen
    if a.workload in gen.RESNET_CONFIGS:
        return resnet_bench(a)

    import numpy as np
    import torch
    from paper_2403_04865_amd import config_from as lib_config
    from paper_2403_04865_amd import SlideLib

    cfg, N = gen.CONFIGS[a.workload]
    if a.tiles:
        N = a.tiles
    ds, ws, ls = gen.SEEDS[a.workload]
    dev = torch.device("cuda:0")
    dtype = 1  # bf16 storage / fp32 accumulate
    recompute = a.recompute if a.recompute >= 0 else int(a.workload == "full")
    lib = SlideLib(lib_config(cfg, dtype, recompute))
    layout = lib.param_layout()
    prm = gen.make_params(cfg, ws)
    flat = np.zeros(lib.slide_param_count(), dtype=np.float32)
    for name, off, ln in layout:
        flat[off:off + ln] = prm[name].reshape(-1)
    params = torch.from_numpy(flat).to(dev)
    grads = torch.zeros_like(params)
    nbytes = lib.slide_chunked_arena_bytes(N, a.chunk_tiles) if a.chunk_tiles else lib.slide_arena_bytes(N)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    o = (-arena.data_ptr()) % 256
    arena = arena[o:o + nbytes]
    lib.slide_bind(params, grads, arena)

    # synthetic slide -> HBM (bf16), generated and uploaded in chunks
    t0 = time.time()
    px = torch.empty((N, 3, cfg.tile, cfg.tile), dtype=torch.bfloat16, device=dev)
    step = 512
    workers = min(16, os.cpu_count() or 1)
    for lo in range(0, N, step):
        hi = min(N, lo + step)
        x = gen.make_pixels(cfg, hi - lo, ds, first_tile=lo, workers=workers)
        px[lo:hi] = torch.from_numpy(x).to(dev).to(torch.bfloat16)
    label = gen.make_label(cfg, ls)
    gen_s = time.time() - t0

    loss = torch.zeros(1, device=dev)
    logits = torch.zeros(cfg.n_classes, device=dev)
    stream = torch.cuda.current_stream()

    def one_step():
        if a.chunk_tiles:   # features of all chunks, pool, then forward again + backward chunk by chunk
            lib.slide_step_chunked(px, N, a.chunk_tiles, label, 0, loss, logits, None, None, stream)
            return
        lib.slide_step_fwd(px, N, label, loss, logits, None, stream)
        lib.slide_step_bwd(0, None, stream)

    for _ in range(a.warmup):
        one_step()
    torch.cuda.synchronize()
    kid = lib.kernel_names().index(a.prof_kernel)
    lib.slide_prof_begin(kid)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k_ms, k_n, k_flops, k_bytes = lib.slide_prof_end()
    peak_alloc = torch.cuda.max_memory_allocated() / 1e9

    ms_per_step = dt / a.steps * 1e3
    tiles_per_s = N * a.steps / dt
    mflops = model_flops_per_tile(cfg) - pruned_flops_per_tile(cfg)   # the bf16 path prunes the last block
    mfu = tiles_per_s * mflops / PEAK["mfma_bf16"]
    stored = load_traffic(a.workload) if not (a.tiles or a.chunk_tiles) else None
    roof = roofline_of(a.prof_kernel, k_ms, k_n, k_flops, k_bytes, dt * 1e3, (stored or {}).get(a.prof_kernel))
    # every family from one more (untimed) step with all launches bracketed by events
    names = lib.kernel_names()
    lib.slide_prof_begin(-1)
    t1 = time.perf_counter()
    one_step()
    torch.cuda.synchronize()
    all_ms = (time.perf_counter() - t1) * 1e3
    lib.slide_prof_end()
    roof_all = []
    for i, nm in enumerate(names):
        f_ms, f_n, f_fl, f_by = lib.slide_prof_family(i)
        if f_n:
            roof_all.append(roofline_of(nm, f_ms, f_n, f_fl, f_by, all_ms, (stored or {}).get(nm)))
    roof_all.sort(key=lambda r: -(r["share_of_step"] or 0))
    traffic_src = None if stored is None else {
        "kind": "stored", "file": f"profiles/traffic_{a.workload}.json", "measured_at_commit": stored.get("_commit"),
        "note": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, scaled by a copy kernel"}

    cpu = None
    if not a.no_cpu_baseline:
        from oracle import slide_oracle as so
        from threadpoolctl import threadpool_info
        nt = a.cpu_tiles
        Xc = px[:nt].float().cpu().numpy().astype(np.float64)
        prm_b = {k: gen.to_bf16_grid(v) for k, v in prm.items()}
        t0 = time.perf_counter()
        so.slide_step(prm_b, Xc, label, cfg, want_pixel_grad=False)
        cs = time.perf_counter() - t0
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        cpu = {"value": round(nt / cs, 3), "unit": "tiles/s", "cores": cores, "kind": "oracle",
               "sample": f"{nt} tiles of the same slide, fp64 numpy oracle, full fwd+bwd step"}

    out = {
        "metric": "tiles/sec fwd+bwd per slide step (1 MI355X); MFMA util % of bf16 peak",
        "value": round(tiles_per_s, 2), "unit": "tiles/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {N} tiles {cfg.tile}x{cfg.tile}x3, ViT dim {cfg.dim} x {cfg.layers} layers "
                               f"x {cfg.heads} heads, gated-attention MIL hidden {cfg.mil_hidden}, {cfg.n_classes} classes",
                   "tiles": N, "slide_steps_per_s": round(a.steps / dt, 4),
                   "model_gflop_per_tile": round(mflops / 1e9, 3), "mfu_bf16_peak": round(mfu, 4),
                   "last_block": "CLS row only after attention (exact; its FLOPs are not counted)",
                   "activation_policy": ("block inputs + re-run blocks in backward" if recompute else "all block activations kept") +
                                        (f"; encoder in chunks of {a.chunk_tiles} tiles (one extra forward)" if a.chunk_tiles else ""),
                   "arena_gb": round(nbytes / 1e9, 2), "peak_alloc_gb_of_288": round(peak_alloc, 2),
                   "loss": float(loss.item()), "input_gen_s": round(gen_s, 1)},
        "roofline": roof,
        "roofline_all": roof_all,
        "traffic_source": traffic_src,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
