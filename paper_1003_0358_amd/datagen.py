"""Seeded synthetic inputs: digit-shaped stroke images and labels.

These stand in for the handwritten-digit benchmark the paper trains on (28x28
uint8 images, background 0, foreground up to 255, content in the central
20x20 box, ten classes).  This module holds no arithmetic of the method itself
(no network, no deformation); the GPU path and its CPU checker both take their
inputs from it.

Recipe for one image: three straight strokes whose end points are uniform in
the central 20x20 box [4,24)^2; every pixel centre within distance 1.0 of a
stroke (width 2) is set to 255; the result is blurred with a separable 7-tap
Gaussian (sigma = 1, taps normalised, zeros outside), rounded to nearest and
clipped to uint8.  Labels are uniform in 0..9 and carry no relation to the
image.  Everything is a pure function of (seed, n).
"""
import numpy as np

H = W = 28
NPIX = H * W
NCLASS = 10


def _blur_taps():
    t = np.arange(-3, 4, dtype=np.float64)
    g = np.exp(-t * t / 2.0)
    return g / g.sum()


def stroke_images(n, seed=0, chunk=4096):
    """-> (images uint8 [n, 784], labels int32 [n])"""
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, NCLASS, size=n, dtype=np.int64).astype(np.int32)
    ends = rng.uniform(4.0, 24.0, size=(n, 3, 2, 2))  # image, stroke, end point, (x, y)
    yy, xx = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    taps = _blur_taps()
    out = np.empty((n, NPIX), dtype=np.uint8)
    for a in range(0, n, chunk):
        e = ends[a:a + chunk]
        m = e.shape[0]
        p0 = e[:, :, 0, :][:, :, None, None, :]           # [m,3,1,1,2]
        p1 = e[:, :, 1, :][:, :, None, None, :]
        d = p1 - p0
        px = np.stack([xx, yy], axis=-1)[None, None]        # [1,1,H,W,2]
        rel = px - p0
        den = np.maximum((d * d).sum(-1), 1e-12)
        t = np.clip((rel * d).sum(-1) / den, 0.0, 1.0)
        near = rel - t[..., None] * d
        dist2 = (near * near).sum(-1)                       # [m,3,H,W]
        img = np.where((dist2 <= 1.0).any(axis=1), 255.0, 0.0)   # [m,H,W]
        # separable blur, zero outside
        pad = np.pad(img, ((0, 0), (0, 0), (3, 3)))
        img = sum(taps[k] * pad[:, :, k:k + W] for k in range(7))
        pad = np.pad(img, ((0, 0), (3, 3), (0, 0)))
        img = sum(taps[k] * pad[:, k:k + H, :] for k in range(7))
        out[a:a + m] = np.clip(np.rint(img), 0, 255).astype(np.uint8).reshape(m, NPIX)
    return out, labels

