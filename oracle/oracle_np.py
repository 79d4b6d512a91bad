"""Second, independent statement of the decode in numpy fp64.  TEST INFRASTRUCTURE ONLY.

Same definition as inr_oracle.c (Sec. III-A/B decode; Sec. IV-A mask; Sec. IV-B
codes; sin frequency w0 from Sec. VI-A), written with array operations: all
pixels of an image at once, each layer one matrix product.  It exists so that
the two oracles can be checked against each other; it shares no code with the C
one or with the GPU library.
"""
from __future__ import annotations

import numpy as np


def dequant(layer) -> np.ndarray:
    if layer.bits == 0:
        w = np.asarray(layer.weights, dtype=np.float32).astype(np.float64)
    else:
        d = np.asarray(layer.weights).astype(np.int64) - int(layer.zp)
        w = (np.float64(np.float32(layer.scale)) * d.astype(np.float64)).astype(np.float32).astype(np.float64)
    if layer.keep is not None:
        w = np.where(np.asarray(layer.keep) != 0, w, 0.0)
    return w.reshape(layer.n_out, layer.n_in)


def decode_image(model, H, W, w0=30.0, lo=-1.0, hi=1.0, clamp=True, affine=None, norm=None) -> np.ndarray:
    """[3, H, W] float64.  affine: None or 6 numbers (2x3 map of the sampling grid, Sec. III-B
    augmentation); norm: None or (scale[3], shift[3]) applied per channel after the clamp."""
    xs = lo + (hi - lo) * (2.0 * np.arange(W) + 1.0) / (2.0 * W)
    ys = lo + (hi - lo) * (2.0 * np.arange(H) + 1.0) / (2.0 * H)
    yy, xx = np.meshgrid(ys, xs, indexing="ij")
    h = np.stack([xx.reshape(-1), yy.reshape(-1)], axis=0)          # [2, H*W], row 0 horizontal
    if affine is not None:
        a = np.asarray(affine, dtype=np.float64).reshape(2, 3)
        h = a[:, :2] @ h + a[:, 2:3]
    n_lin = len(model.layers)
    for l, ly in enumerate(model.layers):
        z = dequant(ly) @ h + np.asarray(ly.bias, dtype=np.float64)[:, None]
        h = np.sin(w0 * z) if l < n_lin - 1 else z
    if clamp:
        h = np.clip(h, 0.0, 1.0)
    if norm is not None:
        h = h * np.asarray(norm[0], dtype=np.float64)[:, None] + np.asarray(norm[1], dtype=np.float64)[:, None]
    return h.reshape(3, H, W)


def decode(models, image_ids, H, W, affine=None, **kw) -> np.ndarray:
    if not len(image_ids):
        return np.zeros((0, 3, H, W))
    return np.stack([decode_image(models[int(i)], H, W, affine=None if affine is None else affine[s], **kw)
                     for s, i in enumerate(image_ids)], axis=0)


def to_u8(c: np.ndarray) -> np.ndarray:
    """round-half-even of 255*c for c already clamped to [0, 1]."""
    return np.rint(255.0 * c).astype(np.uint8)
