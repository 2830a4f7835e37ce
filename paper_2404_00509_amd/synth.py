"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the GPU path's tests/benchmark and the CPU oracle's tests.  It holds none
of the method's arithmetic: only NumPy's seeded generator, image-shaped byte arrays and Gaussian
predictions.  ImageNet-1K itself (Sec. 3 of the paper) is not available; these arrays stand in for
its decoded images with the "maximum side 256" dataset variant of Table 3 and the training
resolutions / batch size of Tables 1 and 9.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    kind: str          # "uniform" (iid bytes, sides in [64,128]) or "gradient" (max side 256)
    out_size: int
    patch: int
    mask_ratio: float
    with_loss: bool
    dtype: str         # "f32" or "bf16": dtype of visible tokens, predictions and gradient

    @property
    def grid(self) -> int:
        return self.out_size // self.patch

    @property
    def L(self) -> int:
        return self.grid * self.grid

    @property
    def D(self) -> int:
        return 3 * self.patch * self.patch


WORKLOADS = {
    "c1": Workload("c1", 64, "uniform", 112, 16, 0.75, False, "f32"),
    "c2": Workload("c2", 256, "gradient", 160, 16, 0.75, False, "f32"),
    "c3": Workload("c3", 1024, "gradient", 192, 16, 0.75, True, "f32"),
    "c4": Workload("c4", 4096, "gradient", 224, 16, 0.75, True, "f32"),
    "c5": Workload("c5", 4096, "gradient", 224, 14, 0.75, True, "bf16"),
}


def image_shapes(kind: str, B: int, seed: int):
    """Heights and widths [B] int32."""
    # one generator per quantity, so that the first B entries do not depend on B
    first = np.random.default_rng([seed, 101, 0])
    second = np.random.default_rng([seed, 101, 1])
    if kind == "uniform":
        h = first.integers(64, 129, size=B)
        w = second.integers(64, 129, size=B)
    elif kind == "gradient":
        other = first.integers(160, 257, size=B)
        landscape = second.integers(0, 2, size=B).astype(bool)
        h = np.where(landscape, other, 256)
        w = np.where(landscape, 256, other)
    elif kind == "gradient500":
        # the "maximum side 500" dataset variants (Table 3; the crop-decode benchmark of Sec. 4.1)
        other = first.integers(313, 501, size=B)
        landscape = second.integers(0, 2, size=B).astype(bool)
        h = np.where(landscape, other, 500)
        w = np.where(landscape, 500, other)
    else:
        raise ValueError(kind)
    return h.astype(np.int32), w.astype(np.int32)


def _one_image(kind: str, h: int, w: int, rng: np.random.Generator) -> np.ndarray:
    if kind == "uniform":
        return rng.integers(0, 256, size=(h, w, 3), dtype=np.uint8)
    base = rng.uniform(40.0, 215.0, size=3)
    gx = rng.uniform(-100.0, 100.0, size=3)
    gy = rng.uniform(-100.0, 100.0, size=3)
    xs = (np.arange(w, dtype=np.float64) / max(w - 1, 1) - 0.5)[None, :, None]
    ys = (np.arange(h, dtype=np.float64) / max(h - 1, 1) - 0.5)[:, None, None]
    noise = rng.integers(-20, 21, size=(h, w, 3))
    v = base[None, None, :] + gx[None, None, :] * xs + gy[None, None, :] * ys + noise
    return np.clip(np.rint(v), 0, 255).astype(np.uint8)


def make_images(kind: str, B: int, seed: int = 0):
    """-> (images uint8 [total], offsets int64 [B], heights int32 [B], widths int32 [B]).

    Image b is HWC, rows tightly packed, starting at images[offsets[b]].  Each image has its own
    generator stream keyed by (seed, b), so image b does not depend on B.
    """
    heights, widths = image_shapes(kind, B, seed)
    sizes = heights.astype(np.int64) * widths.astype(np.int64) * 3
    offsets = np.zeros(B, np.int64)
    offsets[1:] = np.cumsum(sizes)[:-1]
    images = np.empty(int(sizes.sum()), np.uint8)
    for b in range(B):
        rng = np.random.default_rng([seed, 202, b])
        img = _one_image(kind, int(heights[b]), int(widths[b]), rng)
        images[offsets[b]:offsets[b] + sizes[b]] = img.reshape(-1)
    return images, offsets, heights, widths


def image_view(images, offsets, heights, widths, b: int) -> np.ndarray:
    h, w = int(heights[b]), int(widths[b])
    o = int(offsets[b])
    return images[o:o + h * w * 3].reshape(h, w, 3)


def make_pred_rows(seed: int, b: int, L: int, D: int) -> np.ndarray:
    """Predictions ~ N(0,1) for sample b: fp32 [L, D]; keyed by (seed, b) only."""
    rng = np.random.default_rng([seed, 303, b])
    return rng.standard_normal((L, D), dtype=np.float32)


def make_pred(seed: int, B: int, L: int, D: int) -> np.ndarray:
    out = np.empty((B, L, D), np.float32)
    for b in range(B):
        out[b] = make_pred_rows(seed, b, L, D)
    return out


def make_embed_params(seed: int, D: int, E: int, L: int):
    """Parameters of a patch embedding: weight [E, D] ~ N(0, 0.02^2) (the ViT initialisation
    scale), bias [E] ~ N(0, 0.02^2), pos [L, E] uniform in [-1, 1] (the range of the fixed
    sine-cosine positional embedding).  fp32; the caller rounds the weight to bf16."""
    rng = np.random.default_rng([seed, 404, D, E, L])
    weight = (0.02 * rng.standard_normal((E, D))).astype(np.float32)
    bias = (0.02 * rng.standard_normal(E)).astype(np.float32)
    pos = rng.uniform(-1.0, 1.0, (L, E)).astype(np.float32)
    return weight, bias, pos


def make_visible_rows(seed: int, M: int, D: int) -> np.ndarray:
    """Stand-in for visible patch rows when the embedding is tested on its own: image-normalised
    pixel values lie in about [-2.2, 2.7]; uniform over that range, fp32 [M, D]."""
    rng = np.random.default_rng([seed, 505, D])
    return rng.uniform(-2.2, 2.7, (M, D)).astype(np.float32)


def make_ids(seed: int, M: int, L: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 606, L])
    return rng.integers(0, L, M, dtype=np.int32)


def make_jpegs(kind: str, B: int, seed: int = 0, quality: int = 90, subsampling: str = "4:2:0",
               restart_rows: int = 1, optimize: bool = False, restart_blocks: int = 0):
    """The images of make_images(kind, B, seed) as baseline JPEG files (Sec. 4.1: the dataset is
    stored as JPEG at a chosen quality, 90 in the headline configuration), written by the imaging
    library with one restart interval per `restart_rows` rows of MCUs (0: no restart markers, what
    an encoder writes by default) or per `restart_blocks` MCUs.  Returns (files, offsets, sizes):
    the concatenated bytes [sum] uint8, byte offsets [B] int64 and lengths [B] int32."""
    import io

    from PIL import Image

    images, offs, hs, ws = make_images(kind, B, seed)
    chunks, sizes = [], []
    for b in range(B):
        buf = io.BytesIO()
        kw = {} if restart_rows <= 0 else {"restart_marker_rows": restart_rows}
        if restart_blocks > 0:
            kw = {"restart_marker_blocks": restart_blocks}
        Image.fromarray(image_view(images, offs, hs, ws, b)).save(
            buf, format="JPEG", quality=quality, subsampling=subsampling, optimize=optimize, **kw)
        chunks.append(np.frombuffer(buf.getvalue(), np.uint8))
        sizes.append(chunks[-1].size)
    sizes = np.asarray(sizes, np.int32)
    offsets = np.zeros(B, np.int64)
    offsets[1:] = np.cumsum(sizes.astype(np.int64))[:-1]
    return np.concatenate(chunks), offsets, sizes
