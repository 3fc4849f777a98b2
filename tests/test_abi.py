"""Host-side checks that need no GPU: the library loads, exports every symbol slide.h declares,
and its pure-host calls (validation, layout, arena arithmetic) behave as documented."""
import ctypes as C
import os
import re

import pytest

import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2403_04865_amd.binding import lib_path, load_cdll
    if not os.path.exists(lib_path()):
        from paper_2403_04865_amd.build import build
        build()
    return load_cdll()


def test_header_symbols_exported(lib):
    hdr = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b([a-z_0-9]+)\s*\(", hdr)) - {"defined"}
    names = {n for n in names if n.startswith(("slide_", "encoder_", "mil_", "resnet_"))}
    assert {"slide_step_fwd", "slide_step_bwd", "encoder_fwd_tiles", "mil_pool_fwd", "mil_pool_bwd",
            "resnet_slide_step_fwd", "resnet_slide_step_bwd", "resnet_encoder_fwd_tiles"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_layout_matches_generator_names():
    from paper_2403_04865_amd import SlideLib
    from slide_harness import lib_config
    for name in ("tiny", "small", "full"):
        cfg, _ = gen.CONFIGS[name]
        L = SlideLib(lib_config(cfg, 1))
        lay = L.param_layout()
        shapes = gen.param_shapes(cfg)
        assert [n for n, _, _ in lay] == [n for n, _ in shapes]
        off = 0
        for (n, o, ln), (_, shp) in zip(lay, shapes):
            size = 1
            for s in shp:
                size *= s
            assert o == off and ln == size, n
            off += ln
        assert off == L.slide_param_count()
        assert L.slide_param_offset("mil.w") == (lay[-3][1], cfg.mil_hidden)


def test_config_validation():
    from paper_2403_04865_amd import SlideLib, SlideConfig, SlideError
    ok = dict(tile=32, patch=8, dim=64, layers=2, heads=2, mlp_ratio=4, mil_hidden=32, n_classes=1)
    SlideLib(SlideConfig(**ok))
    for bad in (dict(tile=30), dict(heads=3), dict(n_classes=0), dict(dtype=2), dict(layers=-1), dict(ln_eps=0.0),
                dict(recompute=2)):
        with pytest.raises(SlideError) as e:
            SlideLib(SlideConfig(**{**ok, **bad}))
        assert e.value.code == -1
    with pytest.raises(SlideError) as e:
        SlideLib(SlideConfig(**{**ok, "heads": 4}))     # head width 16 is not built
    assert e.value.code == -3


def test_arena_arithmetic_and_unbound_calls(lib):
    from paper_2403_04865_amd import SlideLib, SlideError
    from slide_harness import lib_config
    cfg, _ = gen.CONFIGS["large"]
    L = SlideLib(lib_config(cfg, 1))
    assert L.slide_arena_bytes(0) == 0
    sizes = [L.slide_arena_bytes(n) for n in (1, 16, 256, 8192)]
    assert sizes == sorted(sizes) and sizes[-1] < 288e9
    assert all(s % 256 == 0 for s in sizes)
    assert L.slide_pool_arena_bytes(8192) < sizes[2]
    # block-inputs-only policy: much smaller arena; the 16384-tile ViT-B slide fits one device with it only
    R = SlideLib(lib_config(cfg, 1, recompute=1))
    assert R.slide_arena_bytes(8192) < 0.5 * sizes[-1]
    fcfg, fn = gen.CONFIGS["full"]
    assert SlideLib(lib_config(fcfg, 1, recompute=0)).slide_arena_bytes(fn) > 288e9
    assert SlideLib(lib_config(fcfg, 1, recompute=1)).slide_arena_bytes(fn) + fn * 3 * 224 * 224 * 2 < 270e9
    # nothing bound yet: compute calls refuse without touching the GPU
    with pytest.raises(SlideError) as e:
        L._check(L.lib.slide_step_bwd(L.ctx, 0, None, None), "slide_step_bwd")
    assert e.value.code == -4
    with pytest.raises(SlideError) as e:
        L._check(L.lib.encoder_fwd_tiles(L.ctx, None, 4, None, 0, None), "encoder_fwd_tiles")
    assert e.value.code == -4
    assert L.kernel_names()[0] == "gemm_nt"


def _paper_capacity():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_capacity.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = int(v)
    return out


def test_paper_capacity_arithmetic_and_arena_accounting():
    """The paper's device counts follow from its tiles-per-device figure (Method), and the arena accounting of this
    library (host arithmetic, no GPU) must not need more memory per ViT-B tile than the paper's framework did."""
    import gen
    from paper_2403_04865_amd import SlideLib
    from slide_harness import lib_config
    cap = _paper_capacity()
    k = cap["tiles_per_80GB_vit_base_amp"]
    assert -(-cap["tiles_largest_slide"] // k) == cap["gpus_largest_slide"]
    assert -(-cap["tiles_p99_slide"] // k) == cap["gpus_p99_slide"]
    assert (cap["gpus_finetune_experiment"] - 1) * k == cap["tiles_per_step_finetune_experiment"]
    cfg, _ = gen.CONFIGS["full"]  # ViT-B/16 at 224 px
    lib = SlideLib(lib_config(cfg, 1, 0))  # bf16 storage, every block activation kept
    b1, b2 = lib.slide_arena_bytes(1000), lib.slide_arena_bytes(2000)
    per_tile = (b2 - b1) / 1000.0
    fixed = b1 - 1000 * per_tile
    fits_80 = int((80e9 - fixed) // per_tile)
    assert fits_80 >= k, (fits_80, k)
    # the same accounting puts the paper's largest slide, with per-block recompute, inside one 288 GB device
    lib_r = SlideLib(lib_config(cfg, 1, 1))
    assert lib_r.slide_arena_bytes(16384) < 288e9 < lib.slide_arena_bytes(16384)


def test_resnet_layout_validation_and_arena(lib):
    """Host side of include/resnet.h: tensor order and sizes are those of the generator (and so of the oracle), bad
    shapes are refused, the arena grows with the tile count and the paper's per-device shares fit one device."""
    from paper_2403_04865_amd import ResNetLib, ResNetConfig, SlideError, resnet_config_from
    for name in ("rn_tiny", "rn_tiny_bneck", "rn18", "rn50"):
        cfg, n = gen.RESNET_CONFIGS[name]
        L = ResNetLib(resnet_config_from(cfg))
        assert L.resnet_feature_dim() == cfg.dim
        lay = L.param_layout()
        shapes = gen.resnet_param_shapes(cfg)
        assert [a for a, _, _ in lay] == [a for a, _ in shapes]
        off = 0
        for (nm, o, ln), (_, shp) in zip(lay, shapes):
            size = 1
            for d in shp:
                size *= d
            assert o == off and ln == size, nm
            off += ln
        assert off == L.resnet_param_count()
        assert L.resnet_arena_bytes(0) == 0
        sizes = [L.resnet_arena_bytes(k) for k in (1, max(2, n // 2), n)]
        assert sizes == sorted(sizes) and all(b % 256 == 0 for b in sizes)
        if name in ("rn18", "rn50"):
            # 4,096 ResNet18 tiles (one device's share of the whole-slide breast experiment) and 1,848 ResNet50 tiles
            # (the most the paper fits on 80 GB with 16-bit activations) each fit the 288 GB device with their pixels
            assert sizes[-1] + n * 3 * 224 * 224 * 2 < 270e9, (name, sizes[-1])
    ok = dict(tile=64, block=0, depths=(1, 1, 1, 1), width=64, mil_hidden=32, n_classes=1)
    ResNetLib(ResNetConfig(**ok))
    for bad in (dict(tile=48), dict(block=2), dict(depths=(1, 0, 1, 1)), dict(n_classes=0), dict(bn_eps=0.0)):
        with pytest.raises(SlideError) as e:
            ResNetLib(ResNetConfig(**{**ok, **bad}))
        assert e.value.code == -1
    for bad in (dict(width=8), dict(width=96), dict(width=128, block=1)):
        with pytest.raises(SlideError) as e:
            ResNetLib(ResNetConfig(**{**ok, **bad}))
        assert e.value.code == -3
    L = ResNetLib(ResNetConfig(**ok))
    with pytest.raises(SlideError) as e:
        L._check(L.lib.resnet_slide_step_bwd(L.ctx, 0, None), "resnet_slide_step_bwd")
    assert e.value.code == -4
    assert L.kernel_names()[0] == "conv_fwd"
