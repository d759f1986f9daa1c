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
    mask_mode: str    # "uniform" | "zipf" | "col_aligned" | "aligned"
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


# The paper's own block shapes on MobileNetV1-shaped layers (Section 3.1, Section 5.4): N consecutive
# output channels x one input channel for pointwise convolutions (N = 2, 4, 8 at 70 / 80 / 90 %
# sparsity), and N x (3 x 3) with column origins on multiples of 9 for a 3 x 3 convolution lowered
# to a matrix.  Batch 32.
EXTRA_CONFIGS = (
    LayerConfig("n1", 256, 256, 25088, 2, 1, 0.30, "f16", "uniform", 0.0, "relu_normal",
                1011, 2011, 3011, "MobileNetV1 pointwise 256->256 at 28x28, 2x1 blocks, 70 % sparsity"),
    LayerConfig("n2", 512, 512, 6272, 4, 1, 0.20, "f16", "uniform", 0.0, "relu_normal",
                1012, 2012, 3012, "MobileNetV1 pointwise 512->512 at 14x14, 4x1 blocks, 80 % sparsity"),
    LayerConfig("n3", 1024, 1024, 1568, 8, 1, 0.10, "f16", "uniform", 0.0, "relu_normal",
                1013, 2013, 3013, "MobileNetV1 pointwise 1024->1024 at 7x7, 8x1 blocks, 90 % sparsity"),
    LayerConfig("n4", 256, 2304, 6272, 4, 9, 0.20, "bf16", "col_aligned", 0.0, "relu_normal",
                1014, 2014, 3014, "3x3 convolution 256->256 at 14x14 via im2col, 4x(3x3) blocks, 80 % sparsity"),
)


def aligned_twin(cfg: LayerConfig) -> LayerConfig:
    """The same layer with the same number of blocks at ALIGNED origins (aligned block pruning)."""
    from dataclasses import replace
    return replace(cfg, name=cfg.name + "_abp", mask_mode="aligned", what=cfg.what + " (aligned origins)")


def get_config(name: str) -> LayerConfig:
    for c in CONFIGS + EXTRA_CONFIGS:
        if c.name == name:
            return c
        if c.name + "_abp" == name:
            return aligned_twin(c)
    raise KeyError(name)
