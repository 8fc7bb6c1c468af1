"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it holds none of the method's arithmetic and
is the one piece shared by the CPU oracle's tests and the HIP path's tests / benchmark.

The paper measures on activations of a video diffusion transformer (Wan 2.1 1.3B on
latent grids such as 21x30x52 and 21x45x80, Sec. 4.1 and the implementation table of
the appendix).  Those weights and videos are not available, so these stand-ins keep the
shapes (tokens = T*H*W, 12 heads of 128 channels) and give Q/K/V spatio-temporal
locality by blurring white noise along the three grid axes.
"""
from __future__ import annotations

import numpy as np

__all__ = ["CONFIGS", "iid_normal", "blurred_noise", "make_qkv", "to_bf16_grid"]

# name -> dict(grid, heads, D, dtype, sigma, seed, partitions {kind: (bt,bh,bw,chunk)})
CONFIGS = {
    "tiny": dict(grid=(4, 8, 16), heads=2, D=64, dtype="f32", sigma=0.0, seed=1000,
                 partitions={"1d": (0, 0, 0, 64), "2d": (1, 4, 8, 0), "3d": (2, 4, 4, 0)}),
    "mid": dict(grid=(9, 30, 52), heads=12, D=128, dtype="bf16", sigma=2.0, seed=2000,
                partitions={"3d": (3, 10, 13, 0)}),
    "480p": dict(grid=(21, 30, 52), heads=12, D=128, dtype="bf16", sigma=2.0, seed=3000,
                 # the *_tf entries are the block sizes of the paper's training-free runs at this
                 # resolution (App. A, hyperparameter table): 7 | 24 | 72 blocks
                 partitions={"1d": (0, 0, 0, 1560), "2d": (1, 15, 26, 0), "3d": (3, 15, 13, 0),
                             "1d_tf": (3, 30, 52, 0), "2d_tf": (21, 5, 13, 0), "3d_tf": (7, 5, 13, 0)}),
    "720p": dict(grid=(21, 45, 80), heads=12, D=128, dtype="bf16", sigma=2.0, seed=4000,
                 # *_tf: the paper's block sizes at this resolution (same table): 7 | 40 | 36 blocks
                 partitions={"1d": (0, 0, 0, 2100), "2d": (1, 30, 40, 0), "2d_half": (1, 45, 40, 0),
                             "3d": (3, 15, 40, 0),
                             "1d_tf": (3, 45, 80, 0), "2d_tf": (21, 9, 10, 0), "3d_tf": (7, 15, 20, 0)}),
    # the two latent grids the paper fine-tunes on (93 x 576 x 1024 and 141 x 480 x 832 video), with the block
    # sizes its hyperparameter table gives for them: 8 | 48 | 72 blocks on the first; 3-frame, 5 x 13 and
    # 12 x 10 x 13 blocks on the second, i.e. 12 | 24 | 36 blocks (the table prints 7 for the first of these,
    # which 36 frames in blocks of 3 cannot give)
    "train55k": dict(grid=(24, 36, 64), heads=12, D=128, dtype="bf16", sigma=2.0, seed=6000,
                     partitions={"1d": (3, 36, 64, 0), "2d": (24, 6, 8, 0), "3d": (8, 12, 8, 0)}),
    "train56k": dict(grid=(36, 30, 52), heads=12, D=128, dtype="bf16", sigma=2.0, seed=7000,
                     partitions={"1d": (3, 30, 52, 0), "2d": (36, 5, 13, 0), "3d": (12, 10, 13, 0)}),
    "stress": dict(grid=(31, 45, 80), heads=40, D=128, dtype="bf16", sigma=(1.0, 4.0, 16.0),
                   seed=5000, partitions={"3d": (3, 15, 16, 0)}),
}


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return them as
    float32, so the CPU and the GPU side can be fed bit-identical numbers."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def iid_normal(seed: int, shape) -> np.ndarray:
    """iid N(0,1) float32 tensor from numpy's default_rng(seed)."""
    return np.random.default_rng(seed).standard_normal(shape, dtype=np.float32)


def blurred_noise(seed: int, grid, heads: int, D: int, sigma, batch: int = 1) -> np.ndarray:
    """White noise on the T x H x W grid, Gaussian-blurred along all three axes
    (sigma in tokens, kernel truncated at 4 sigma, reflecting boundary), independently for
    every (batch, head, channel), then standardised to mean 0 / std 1 over the tensor.
    sigma may be a tuple: head h uses sigma[h % len(sigma)].  Returns [B, S, heads, D]."""
    from scipy.ndimage import gaussian_filter1d

    T, H, W = grid
    rng = np.random.default_rng(seed)
    sig = sigma if isinstance(sigma, (tuple, list)) else (sigma,)
    out = np.empty((batch, T * H * W, heads, D), dtype=np.float32)
    for b in range(batch):
        for h in range(heads):
            f = rng.standard_normal((T, H, W, D), dtype=np.float32)
            s = float(sig[h % len(sig)])
            if s > 0:
                for ax in range(3):
                    f = gaussian_filter1d(f, s, axis=ax, mode="reflect", truncate=4.0)
            out[b, :, h, :] = f.reshape(T * H * W, D)
    out -= out.mean(dtype=np.float64)
    out /= out.std(dtype=np.float64)
    return out


def make_qkv(name: str, with_dO: bool = True, heads: int | None = None):
    """Q, K, V (and dO) of a named configuration, caller layout [1, S, heads, D], float32
    holding values exactly representable in the configuration's dtype."""
    c = CONFIGS[name]
    Hh = heads if heads is not None else c["heads"]
    T, H, W = c["grid"]
    n = 4 if with_dO else 3
    ts = []
    for i in range(n):
        if c["sigma"] == 0.0:
            x = iid_normal(c["seed"] + i, (1, T * H * W, Hh, c["D"]))
        else:
            x = blurred_noise(c["seed"] + i, c["grid"], Hh, c["D"], c["sigma"])
        if c["dtype"] == "bf16":
            x = to_bf16_grid(x)
        ts.append(x)
    return ts
