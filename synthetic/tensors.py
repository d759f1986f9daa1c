"""Seeded dense weights / activations and their 16-bit encodings.

Values are drawn in float32 with numpy's default_rng and rounded once (to nearest,
ties to even) to the layer's element type.  Both the oracle side and the HIP side of
every test receive these already-rounded values: `encode` gives the bit patterns handed
to the device, `decode_f64` the exact same values as float64 for the oracle.
"""
import numpy as np

from .configs import LayerConfig
from .masks import select_blocks

_NP = {"f32": np.float32, "f16": np.float16}


def encode(a32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> array holding the element type's bits (f32 / f16 / uint16 for bf16)."""
    a32 = np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == "f32":
        return a32
    if dtype == "f16":
        return a32.astype(np.float16)
    if dtype == "bf16":
        u = a32.view(np.uint32).astype(np.uint64)
        lsb = (u >> 16) & 1
        u = (u + 0x7FFF + lsb) >> 16          # round to nearest even (finite inputs)
        return u.astype(np.uint16)
    raise ValueError(dtype)


def decode_f64(enc: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of every encoded element."""
    if dtype in ("f32", "f16"):
        return enc.astype(np.float64)
    if dtype == "bf16":
        return (enc.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def make_weights(M, K, seed, dtype):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((M, K), dtype=np.float32) * np.float32(np.sqrt(2.0 / K))
    return encode(w, dtype)


def make_activations(K, N, seed, dtype, dist):
    rng = np.random.default_rng(seed)
    if dist == "uniform01":
        x = rng.random((K, N), dtype=np.float32)
    elif dist == "relu_normal":
        x = np.maximum(rng.standard_normal((K, N), dtype=np.float32), np.float32(0))
    elif dist == "normal":
        x = rng.standard_normal((K, N), dtype=np.float32)
    else:
        raise ValueError(dist)
    return encode(x, dtype)


def make_layer(cfg: LayerConfig, N=None):
    """(blocks[nb,2] int32, W encoded [M,K], X encoded [K,N]) for a layer config."""
    n = cfg.N if N is None else N
    blocks = select_blocks(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed,
                           cfg.mask_mode, cfg.zipf_s)
    W = make_weights(cfg.M, cfg.K, cfg.w_seed, cfg.dtype)
    X = make_activations(cfg.K, n, cfg.x_seed, cfg.dtype, cfg.x_dist)
    return blocks, W, X
