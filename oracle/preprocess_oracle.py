"""CPU oracle for GPU-side image preprocessing.  TEST INFRASTRUCTURE ONLY.

Only tests may import this module; the product path never does, and this module imports nothing
from the product.

What it computes.  The paper (Sec. 2, "Image Preprocessing") lists the steps that precede the
encoder: (1) resize, rescale, pad and normalise the raw image, (2) segment it into tiles,
(3) tile-level transformations and sampling; the number of tiles grows with the image size (an
896 x 896 image gives 4, 5 or 10 tiles for the models of Table 1).  It gives no formulas, so the
steps are taken in their plainest form, written out in float64:

  * resize to (grid_rows * S) x (grid_cols * S) by bilinear interpolation with pixel centres at
    half-integers: source coordinate of output pixel o is (o + 0.5) * (in / out) - 0.5, clamped
    below at 0; the two taps are floor(.) and the next pixel (the last pixel repeats at the edge);
    no low-pass filter when shrinking;
  * rescale 8-bit values by 1/255, normalise per channel: (v - mean[c]) / std[c];
  * cut the resized image into grid_rows * grid_cols tiles of S x S, tile order row-major, each tile
    channel-first [C, S, S]: the layout the encoder takes;
  * optionally one more tile, last: the whole image resized to S x S ("thumbnail", the extra tile
    behind Table 1's 5 = 4 + 1 tiles).
Padding, step (3) and the choice of the tile grid from the image size are not modelled: the grid is
an argument.

Pins (tests/test_oracle_preprocess.py): same-size resize is the identity; a constant image stays
constant; an image that is linear in x and y is reproduced exactly away from the clamped border;
torch.nn.functional.interpolate(mode="bilinear", align_corners=False) as a library second opinion;
the normalisation closed form; the tile order by brute force.
"""
from __future__ import annotations

import numpy as np


def resize_bilinear(img: np.ndarray, out_h: int, out_w: int) -> np.ndarray:
    """img [H, W, C] (any real dtype) -> [out_h, out_w, C] float64."""
    img = np.asarray(img, dtype=np.float64)
    H, W, _ = img.shape

    def taps(n_in, n_out):
        src = (np.arange(n_out, dtype=np.float64) + 0.5) * (n_in / n_out) - 0.5
        src = np.maximum(src, 0.0)
        i0 = np.minimum(np.floor(src).astype(np.int64), n_in - 1)
        i1 = np.minimum(i0 + 1, n_in - 1)
        return i0, i1, src - i0

    y0, y1, wy = taps(H, out_h)
    x0, x1, wx = taps(W, out_w)
    out = np.empty((out_h, out_w, img.shape[2]), dtype=np.float64)
    for oy in range(out_h):
        top = img[y0[oy]][x0] * (1.0 - wx)[:, None] + img[y0[oy]][x1] * wx[:, None]
        bot = img[y1[oy]][x0] * (1.0 - wx)[:, None] + img[y1[oy]][x1] * wx[:, None]
        out[oy] = top * (1.0 - wy[oy]) + bot * wy[oy]
    return out


def normalize(img: np.ndarray, mean, std) -> np.ndarray:
    """8-bit scale to [0, 1], then (v - mean[c]) / std[c] per channel; img [..., C]."""
    return (np.asarray(img, dtype=np.float64) / 255.0 - np.asarray(mean, dtype=np.float64)) / np.asarray(std, dtype=np.float64)


def preprocess_tiles(img_u8: np.ndarray, S: int, grid_rows: int, grid_cols: int, thumbnail: bool, mean, std) -> np.ndarray:
    """img_u8 [H, W, C] uint8 -> [grid_rows*grid_cols (+1), C, S, S] float64."""
    if img_u8.dtype != np.uint8 or img_u8.ndim != 3:
        raise ValueError("image must be [H, W, C] uint8")
    if grid_rows < 1 or grid_cols < 1 or S < 1:
        raise ValueError("grid and tile size must be positive")
    big = normalize(resize_bilinear(img_u8, grid_rows * S, grid_cols * S), mean, std)
    tiles = []
    for ty in range(grid_rows):
        for tx in range(grid_cols):
            tiles.append(big[ty * S:(ty + 1) * S, tx * S:(tx + 1) * S].transpose(2, 0, 1))
    if thumbnail:
        tiles.append(normalize(resize_bilinear(img_u8, S, S), mean, std).transpose(2, 0, 1))
    return np.stack(tiles)
