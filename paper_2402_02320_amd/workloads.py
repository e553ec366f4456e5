"""Seeded synthetic inputs for the five benchmark configurations.

This module holds NO protocol arithmetic: it only draws plaintext real-valued
tensors with numpy's seeded generator and rearranges them (im2col).  Encoding,
sharing, triples and truncation tuples are produced separately by the GPU
library and, independently, by the test oracle.  The tensors stand in for the
paper's MNIST / CIFAR10 / ImageNet workloads (Section 8.3 and 8.4), from which
only the shapes are taken.
"""
from dataclasses import dataclass

import numpy as np

SEED_BASE = 0x5350494E00  # "SPIN" << 8; config c uses SEED_BASE + c


@dataclass(frozen=True)
class GemmShape:
    name: str
    batch: int
    M: int
    N: int
    K: int


@dataclass(frozen=True)
class Config:
    cfg: int
    n: int                      # parties
    f: int                      # fractional bits
    dist: str                   # plaintext distribution
    gemms: tuple                # GemmShape entries
    vec: int = 0                # length of the elementwise Beaver mul (0 = none)
    note: str = ""

    @property
    def seed(self):
        return SEED_BASE + self.cfg


CONFIGS = {
    1: Config(1, 3, 16, "uniform(-1,1)", (GemmShape("xy", 1, 64, 64, 64),),
              note="latency / parity case"),
    2: Config(2, 2, 16, "normal(0,1)", (GemmShape("xy", 1, 1024, 1024, 1024),), vec=1 << 24,
              note="square GEMM + 2^24-element Beaver mul + truncation"),
    3: Config(3, 3, 16, "normal(0,0.1)", (GemmShape("conv_im2col", 1, 131072, 64, 576),),
              note="batch 128, 3x3 conv 64->64 on 32x32 maps as an im2col GEMM "
                   "(the third conv layer of the paper's VGG16 variant, Appendix A)"),
    4: Config(4, 3, 16, "normal(0,1)",
              (GemmShape("qkT", 64, 128, 128, 64), GemmShape("pv", 64, 128, 64, 128)), vec=1 << 20,
              note="8 batch x 8 heads attention GEMMs (Section 7.4) + elementwise mul on scores"),
    5: Config(5, 5, 16, "uniform(-4,4)", (GemmShape("xy", 1, 4096, 4096, 4096),),
              note="headline: open + share update + truncation end to end"),
}


def _draw(rng, dist, shape):
    if dist == "uniform(-1,1)":
        return rng.uniform(-1.0, 1.0, size=shape)
    if dist == "uniform(-4,4)":
        return rng.uniform(-4.0, 4.0, size=shape)
    if dist == "normal(0,1)":
        return rng.normal(0.0, 1.0, size=shape)
    if dist == "normal(0,0.1)":
        return rng.normal(0.0, 0.1, size=shape)
    raise ValueError(dist)


def im2col_3x3(fmap):
    """[B,C,H,W] -> [B*H*W, C*9] patches of a 3x3, stride 1, zero-pad 1 convolution."""
    B, C, H, W = fmap.shape
    padded = np.zeros((B, C, H + 2, W + 2), dtype=fmap.dtype)
    padded[:, :, 1:-1, 1:-1] = fmap
    win = np.lib.stride_tricks.sliding_window_view(padded, (3, 3), axis=(2, 3))  # B,C,H,W,3,3
    return np.ascontiguousarray(win.transpose(0, 2, 3, 1, 4, 5)).reshape(B * H * W, C * 9)


def gemm_plaintexts(cfg, gemm_index=0, scale=1.0):
    """Real-valued X [batch,M,K] and Y [batch,K,N] of one GEMM of a configuration.

    scale < 1 shrinks the batch-like dimension (M for single GEMMs, the image
    batch for the conv case, `batch` for the attention case) for quick tests;
    the shape actually produced is read off the returned arrays."""
    c = CONFIGS[cfg]
    g = c.gemms[gemm_index]
    rng = np.random.default_rng(c.seed * 16 + gemm_index)
    if g.name == "conv_im2col":
        images = max(1, int(round(128 * scale)))
        fmap = _draw(rng, c.dist, (images, 64, 32, 32))
        X = im2col_3x3(fmap)[None]                       # [1, images*1024, 576]
        Y = _draw(rng, c.dist, (1, g.K, g.N))
        return X, Y
    batch = g.batch if g.batch == 1 else max(1, int(round(g.batch * scale)))
    M = g.M if g.batch > 1 else max(1, int(round(g.M * scale)))
    X = _draw(rng, c.dist, (batch, M, g.K))
    Y = _draw(rng, c.dist, (batch, g.K, g.N))
    return X, Y


def vec_plaintexts(cfg, count=None):
    """Two real-valued vectors for the elementwise Beaver multiplication."""
    c = CONFIGS[cfg]
    count = c.vec if count is None else count
    rng = np.random.default_rng(c.seed * 16 + 8)
    return _draw(rng, c.dist, (count,)), _draw(rng, c.dist, (count,))
