"""The five synthetic layer shapes the build is measured on.

They stand in for the ImageNet-trained MobileNet / ResNet layers the paper measures
(Section 5.1, Section 5.4): same GEMM shapes, He-initialised weights, post-ReLU-like
activations and seeded random unaligned block masks.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class LayerConfig:
    name: str
    M: int            # output channels (rows of W, rows of Y)
    K: int            # input channels x kernel taps (columns of W, rows of X)
    N: int            # pixels x batch (columns of X and Y)
    bh: int           # block height (consecutive output channels)
    bw: int           # block width (consecutive input channels)
    density: float    # kept fraction of W's elements (1 - pruning rate)
    dtype: str        # "f32" | "f16" | "bf16"  (input element type)
    mask_mode: str    # "uniform" | "zipf"
    zipf_s: float     # Zipf exponent over bh-row stripes (zipf mode only)
    x_dist: str       # "uniform01" | "relu_normal" | "normal"
    mask_seed: int
    w_seed: int
    x_seed: int
    what: str


CONFIGS = (
    LayerConfig("c0", 64, 64, 196, 4, 4, 0.50, "f32", "uniform", 0.0, "uniform01",
                1000, 2000, 3000, "tiny layer, one 14x14 map"),
    LayerConfig("c1", 960, 160, 1568, 4, 4, 0.30, "f16", "uniform", 0.0, "relu_normal",
                1001, 2001, 3001, "MobileNetV2-style pointwise conv, batch 32 x 7x7"),
    LayerConfig("c2", 1024, 256, 12544, 8, 8, 0.20, "f16", "uniform", 0.0, "relu_normal",
                1002, 2002, 3002, "ResNet-50 bottleneck 1x1 expand, batch 64 x 14x14"),
    LayerConfig("c3", 256, 2304, 12544, 4, 4, 0.25, "bf16", "uniform", 0.0, "relu_normal",
                1003, 2003, 3003, "ResNet-50 3x3 conv via im2col, batch 64 x 14x14"),
    LayerConfig("c4", 4096, 4096, 8192, 16, 16, 0.10, "bf16", "zipf", 1.1, "normal",
                1004, 2004, 3004, "roofline-stress layer, Zipf-skewed stripes"),
)


def get_config(name: str) -> LayerConfig:
    for c in CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)
