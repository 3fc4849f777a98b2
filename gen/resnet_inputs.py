"""Seeded synthetic weights for the convolutional tile encoders (ResNet family).

The paper's experiments train ResNet18 and ResNet50 tile encoders under a gated-attention
aggregator (Results: gradient-equivalence experiment, EGFR experiment, whole-slide breast
experiment: ResNet18 on 4,096 tiles of 224 px per device).  This module only names the tensors
of such a network, gives their shapes and draws them from seeded streams; pixels and labels
come from slide_inputs.  No convolution, normalisation, pooling or gradient arithmetic here.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np


@dataclass(frozen=True)
class ResNetConfig:
    tile: int            # S: tile side in pixels (a multiple of 32)
    block: str           # "basic" (two 3x3 convolutions) or "bottleneck" (1x1, 3x3, 1x1 with 4x expansion)
    depths: tuple        # blocks per stage, four stages
    width: int           # channels of the stem and the first stage (64); stage s has width * 2^s
    mil_hidden: int      # M_h of the gated-attention aggregator
    n_classes: int       # C: 1 -> one logit + BCE, >1 -> softmax cross-entropy
    bn_eps: float = 1e-5

    @property
    def expansion(self) -> int:
        return 1 if self.block == "basic" else 4

    @property
    def dim(self) -> int:      # feature width behind the global average pool
        return self.width * 8 * self.expansion

    def as_dict(self):
        return asdict(self)


RESNET_CONFIGS = {
    # brute-force sized
    "rn_probe": (ResNetConfig(32, "basic", (1, 1, 1, 1), 8, 4, 1), 3),
    # every kernel shape class at a size the oracle finishes in seconds
    "rn_tiny": (ResNetConfig(64, "basic", (1, 1, 1, 1), 64, 32, 1), 6),
    "rn_tiny_bneck": (ResNetConfig(64, "bottleneck", (1, 1, 1, 1), 64, 32, 4), 5),
    # ResNet18 / ResNet50 as in the paper's experiments; 4096 tiles of 224 px is one device's share of the whole-slide
    # breast experiment
    "rn18_small": (ResNetConfig(224, "basic", (2, 2, 2, 2), 64, 128, 1), 8),
    "rn18": (ResNetConfig(224, "basic", (2, 2, 2, 2), 64, 128, 1), 4096),
    "rn50_small": (ResNetConfig(224, "bottleneck", (3, 4, 6, 3), 64, 128, 1), 4),
    "rn50": (ResNetConfig(224, "bottleneck", (3, 4, 6, 3), 64, 128, 1), 1848),
}

RESNET_SEEDS = {
    "rn_probe": (1100, 2100, 3100),
    "rn_tiny": (1101, 2101, 3101),
    "rn_tiny_bneck": (1102, 2102, 3102),
    "rn18_small": (1103, 2103, 3103),
    "rn18": (1104, 2103, 3104),
    "rn50_small": (1105, 2105, 3105),
    "rn50": (1106, 2105, 3106),
}


def resnet_blocks(cfg: ResNetConfig):
    """Ordered list of residual blocks: dict(name, cin, mid, cout, stride, down)."""
    out = []
    cin = cfg.width
    for s, depth in enumerate(cfg.depths):
        mid = cfg.width * (2 ** s)
        cout = mid * cfg.expansion
        for b in range(depth):
            stride = 2 if (b == 0 and s > 0) else 1
            down = stride != 1 or cin != cout
            out.append(dict(name=f"s{s}.b{b}", cin=cin, mid=mid, cout=cout, stride=stride, down=down))
            cin = cout
    return out


def resnet_param_shapes(cfg: ResNetConfig):
    """Ordered (name, shape) list of every trainable tensor.  Convolution weights are
    [out][in][kh][kw]; convolutions carry no bias (each is followed by a batch normalisation)."""
    w = cfg.width
    out = [("stem.conv.W", (w, 3, 7, 7)), ("stem.bn.g", (w,)), ("stem.bn.b", (w,))]
    for blk in resnet_blocks(cfg):
        p = blk["name"] + "."
        cin, mid, cout = blk["cin"], blk["mid"], blk["cout"]
        if cfg.block == "basic":
            out += [(p + "conv1.W", (mid, cin, 3, 3)), (p + "bn1.g", (mid,)), (p + "bn1.b", (mid,)),
                    (p + "conv2.W", (cout, mid, 3, 3)), (p + "bn2.g", (cout,)), (p + "bn2.b", (cout,))]
        else:
            out += [(p + "conv1.W", (mid, cin, 1, 1)), (p + "bn1.g", (mid,)), (p + "bn1.b", (mid,)),
                    (p + "conv2.W", (mid, mid, 3, 3)), (p + "bn2.g", (mid,)), (p + "bn2.b", (mid,)),
                    (p + "conv3.W", (cout, mid, 1, 1)), (p + "bn3.g", (cout,)), (p + "bn3.b", (cout,))]
        if blk["down"]:
            out += [(p + "down.conv.W", (cout, cin, 1, 1)), (p + "down.bn.g", (cout,)), (p + "down.bn.b", (cout,))]
    D, Mh, C = cfg.dim, cfg.mil_hidden, cfg.n_classes
    out += [("mil.V.W", (Mh, D)), ("mil.V.b", (Mh,)), ("mil.U.W", (Mh, D)), ("mil.U.b", (Mh,)), ("mil.w", (Mh,)),
            ("head.W", (C, D)), ("head.b", (C,))]
    return out


def make_resnet_params(cfg: ResNetConfig, seed: int):
    """dict name -> float32 array.

    Convolution weights ~ N(0, 2 / (out_channels * kh * kw)) (the usual fan-out law for ReLU
    networks); batch-norm gains 1 + N(0, 0.1^2) and shifts N(0, 0.1^2), so that no test passes with
    a gain or shift dropped; aggregator matrices N(0, 0.05^2) with draws beyond two standard deviations
    redrawn, aggregator biases N(0, 0.02^2).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, shape in resnet_param_shapes(cfg):
        leaf = name.split(".")[-1]
        if name.startswith(("mil.", "head.")):
            std = 0.02 if leaf == "b" else 0.05
            x = rng.standard_normal(shape)
            bad = np.abs(x) > 2.0
            while bad.any():
                x[bad] = rng.standard_normal(int(bad.sum()))
                bad = np.abs(x) > 2.0
            v = x * std
        elif leaf == "W":
            fan_out = shape[0] * shape[2] * shape[3]
            v = rng.standard_normal(shape) * np.sqrt(2.0 / fan_out)
        elif leaf == "g":
            v = 1.0 + 0.1 * rng.standard_normal(shape)
        else:
            v = 0.1 * rng.standard_normal(shape)
        out[name] = v.astype(np.float32)
    return out
