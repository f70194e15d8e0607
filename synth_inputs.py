"""Seeded synthetic descriptor maps shaped like a dense matching head's output.

This module only *generates inputs* (and the seed grid); it contains none of the
matching method's arithmetic, so both the CPU oracle's tests and the GPU path's
tests may import it.  Everything is a pure function of its integer seed.

The maps stand in for the per-pixel descriptor maps D1, D2 of shape H x W x d
that the matching head produces (paper section 3.2.4, "Matching Head"); the paper
evaluates on public indoor/outdoor image-pair benchmarks with pretrained
weights, neither of which is used here.

Layout returned everywhere: row-major ``[H*W][d]`` float32, pixel id ``y*W+x``.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "exact_pair",
    "gaussian_map",
    "random_homography",
    "warped_pair",
    "grid_seeds",
    "config_shape",
    "config_pair",
]


def exact_pair(seed: int, width: int = 64, height: int = 48, d: int = 24):
    """Two independent maps whose entries are k/8, k uniform integer in [-8, 8].

    Every product is a multiple of 1/64 and every dot product of d<=64 terms is
    exactly representable in fp16-input/fp32-accumulate, fp32 and fp64
    arithmetic, so any correct implementation returns identical bits and ties
    (which are frequent) are decided purely by the tie-break rule.
    """
    rng = np.random.default_rng(seed)
    n = width * height
    a = rng.integers(-8, 9, size=(n, d)).astype(np.float32) / np.float32(8.0)
    b = rng.integers(-8, 9, size=(n, d)).astype(np.float32) / np.float32(8.0)
    return a, b


def _l2_normalise(x: np.ndarray) -> np.ndarray:
    nrm = np.sqrt((x * x).sum(axis=-1, keepdims=True))
    return x / nrm


def gaussian_map(rng: np.random.Generator, width: int, height: int, d: int) -> np.ndarray:
    """i.i.d. N(0,1) per channel, L2-normalised per pixel (float64)."""
    return _l2_normalise(rng.standard_normal((height * width, d)))


def _dlt_homography(src: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """3x3 H with dst ~ H * src from four point pairs (direct linear transform)."""
    rows = []
    for (x, y), (u, v) in zip(src, dst):
        rows.append([-x, -y, -1.0, 0.0, 0.0, 0.0, u * x, u * y, u])
        rows.append([0.0, 0.0, 0.0, -x, -y, -1.0, v * x, v * y, v])
    a = np.asarray(rows, dtype=np.float64)
    _, _, vt = np.linalg.svd(a)
    h = vt[-1].reshape(3, 3)
    return h / h[2, 2]


def random_homography(rng: np.random.Generator, width: int, height: int, jitter: float = 0.15) -> np.ndarray:
    """Homography moving the four image corners by U(-jitter, jitter) * (W, H)."""
    corners = np.array(
        [[0.0, 0.0], [width - 1.0, 0.0], [width - 1.0, height - 1.0], [0.0, height - 1.0]]
    )
    shift = rng.uniform(-jitter, jitter, size=(4, 2)) * np.array([width, height], dtype=np.float64)
    return _dlt_homography(corners, corners + shift)


def warped_pair(seed: int, width: int = 512, height: int = 384, d: int = 24,
                noise_std: float = 0.1, jitter: float = 0.15):
    """Map 1: normalised Gaussian.  Map 2: map 1 seen through a random homography.

    Pixel (x, y) of map 2 samples map 1 bilinearly at H*(x, y, 1) (backward
    warp); a sample point outside [0, W-1] x [0, H-1] receives a fresh N(0,1)
    vector instead; N(0, noise_std) noise is added per channel and every pixel
    is renormalised.  Returns (map1, map2, H) with the maps as float32.
    """
    rng = np.random.default_rng(seed)
    m1 = gaussian_map(rng, width, height, d)
    hmat = random_homography(rng, width, height, jitter)

    ys, xs = np.meshgrid(np.arange(height, dtype=np.float64), np.arange(width, dtype=np.float64), indexing="ij")
    pts = np.stack([xs.ravel(), ys.ravel(), np.ones(width * height)], axis=0)
    wp = hmat @ pts
    sx = wp[0] / wp[2]
    sy = wp[1] / wp[2]
    inside = (wp[2] > 0) & (sx >= 0.0) & (sx <= width - 1.0) & (sy >= 0.0) & (sy <= height - 1.0)

    sxc = np.clip(np.where(inside, sx, 0.0), 0.0, width - 1.0)
    syc = np.clip(np.where(inside, sy, 0.0), 0.0, height - 1.0)
    x0 = np.minimum(np.floor(sxc).astype(np.int64), width - 2)
    y0 = np.minimum(np.floor(syc).astype(np.int64), height - 2)
    fx = (sxc - x0)[:, None]
    fy = (syc - y0)[:, None]
    i00 = y0 * width + x0
    m2 = ((1 - fx) * (1 - fy) * m1[i00] + fx * (1 - fy) * m1[i00 + 1]
          + (1 - fx) * fy * m1[i00 + width] + fx * fy * m1[i00 + width + 1])
    fresh = rng.standard_normal((height * width, d))
    m2 = np.where(inside[:, None], m2, fresh)
    m2 = m2 + rng.normal(0.0, noise_std, size=m2.shape)
    m2 = _l2_normalise(m2)
    return m1.astype(np.float32), m2.astype(np.float32), hmat


def grid_seeds(width: int, height: int, subsample: int = 8) -> np.ndarray:
    """Flat pixel ids of the grid x in {0, s, 2s, ...}, y in {0, s, 2s, ...} (phase 0)."""
    ys = np.arange(0, height, subsample, dtype=np.int64)
    xs = np.arange(0, width, subsample, dtype=np.int64)
    return (ys[:, None] * width + xs[None, :]).reshape(-1).astype(np.int32)


# The five workload shapes: (width, height, d, pairs in the batch).
_CONFIG_SHAPES = {
    1: (64, 48, 24, 1),
    2: (512, 384, 24, 1),
    3: (512, 384, 24, 1),
    4: (512, 384, 24, 16),
    5: (1024, 768, 24, 1),
}


def config_shape(cfg: int):
    return _CONFIG_SHAPES[cfg]


def config_pair(cfg: int, pair_index: int = 0):
    """The (map1, map2) pair of workload configuration ``cfg`` (1..5).

    Configuration 3 reuses configuration 2's pair (same seed); the seed of a
    pair is 1000*cfg + pair_index.
    """
    width, height, d, _ = _CONFIG_SHAPES[cfg]
    if cfg == 1:
        return exact_pair(1000 + pair_index, width, height, d)
    base = 2 if cfg == 3 else cfg
    m1, m2, _ = warped_pair(1000 * base + pair_index, width, height, d)
    return m1, m2
