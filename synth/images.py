"""Seeded synthetic uint8 images (stand-ins for CIFAR-10 / Caltech-101 inputs).

Config 0 uses uniform random pixels.  The other configs use smooth random
fields: uniform noise blurred by a separable 3-tap [1,2,1]/4 kernel (edge
replicated) and stretched to the full 0..255 range.  Image `item` (1-based) of
workload `config` is drawn from PCG64(1000*config + item).
"""
from __future__ import annotations

import numpy as np

from .models import CONFIGS


def make_image(config: int, item: int = 1, shape: tuple | None = None) -> np.ndarray:
    """uint8 array [C][H][W] for image number `item` >= 1 of workload `config`."""
    assert item >= 1
    c, h, w = shape or CONFIGS[config]["shape"]
    rng = np.random.Generator(np.random.PCG64(1000 * config + item))
    if config == 0:
        return rng.integers(0, 256, size=(c, h, w), dtype=np.int64).astype(np.uint8)
    f = rng.random(size=(c, h, w))
    for axis in (1, 2):
        p = np.concatenate([np.take(f, [0], axis=axis), f, np.take(f, [-1], axis=axis)], axis=axis)
        n = f.shape[axis]
        lo = np.take(p, range(0, n), axis=axis)
        mid = np.take(p, range(1, n + 1), axis=axis)
        hi = np.take(p, range(2, n + 2), axis=axis)
        f = 0.25 * lo + 0.5 * mid + 0.25 * hi
    fmin, fmax = f.min(), f.max()
    img = np.rint((f - fmin) / (fmax - fmin) * 255.0)
    return np.clip(img, 0, 255).astype(np.uint8)
