"""Seeded synthetic images standing in for down-sampled natural images.

"filtered": white Gaussian noise, blurred per channel with a separable Gaussian
(sigma 2 px, radius 6, circular boundary), normalised per image to mean 128 and
standard deviation 50, rounded half away from zero and clipped to [0, 255]. The
blur gives the neighbouring-pixel correlation of a natural image at these sizes.
"uniform": independent bytes, uniform on [0, 255].
"""
import numpy as np

from . import prng


def _blur_kernel(sigma=2.0, radius=6):
    t = np.arange(-radius, radius + 1, dtype=np.float64)
    k = np.exp(-0.5 * (t / sigma) ** 2)
    return k / k.sum()


def _blur_axis(a, k, axis):
    r = (len(k) - 1) // 2
    out = np.zeros_like(a)
    for i, kv in enumerate(k):
        out += kv * np.roll(a, i - r, axis=axis)
    return out


def make_images(cfg, batch=None, seed=None, kind=None):
    """uint8 array [batch, 3, H, W] for configuration `cfg`."""
    b = cfg.batch if batch is None else batch
    seed = (1000 + cfg.seed_id) if seed is None else seed
    kind = cfg.image_kind if kind is None else kind
    n = b * 3 * cfg.H * cfg.W
    if b == 0:
        return np.zeros((0, 3, cfg.H, cfg.W), dtype=np.uint8)
    if kind == "uniform":
        v = prng.randint(prng.substream(seed, 1), n, 0, 256)
        return v.astype(np.uint8).reshape(b, 3, cfg.H, cfg.W)
    g = prng.normal(prng.substream(seed, 2), n).reshape(b, 3, cfg.H, cfg.W)
    k = _blur_kernel()
    g = _blur_axis(_blur_axis(g, k, 2), k, 3)
    g = g - g.mean(axis=(1, 2, 3), keepdims=True)
    g = g / g.std(axis=(1, 2, 3), keepdims=True)
    g = g * 50.0 + 128.0
    g = np.sign(g) * np.floor(np.abs(g) + 0.5)
    return np.clip(g, 0, 255).astype(np.uint8)


def make_large_image(h, w, seed=1900):
    """One planar uint8 image [3, h, w] of the "filtered" kind, standing in for a high-resolution
    photograph that is coded patch by patch."""
    from types import SimpleNamespace
    return make_images(SimpleNamespace(batch=1, seed_id=0, image_kind="filtered", H=h, W=w), batch=1, seed=seed)[0]
