"""Pins for the preprocessing oracle (Sec. 2, "Image Preprocessing"): closed forms, invariants, a library routine."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import gen
from oracle import preprocess_oracle as P

MEAN, STD = (0.48, 0.45, 0.41), (0.27, 0.26, 0.28)


def test_same_size_resize_is_identity_and_constant_stays_constant():
    img = gen.make_image_u8(13, 17, 3, seed=0)
    np.testing.assert_array_equal(P.resize_bilinear(img, 13, 17), img.astype(np.float64))
    flat = np.full((9, 5, 3), 77, dtype=np.uint8)
    for oh, ow in [(4, 4), (9, 5), (20, 31)]:
        np.testing.assert_allclose(P.resize_bilinear(flat, oh, ow), 77.0, rtol=0, atol=1e-12)


@pytest.mark.parametrize("H,W,oh,ow", [(8, 12, 16, 24), (8, 12, 20, 30), (30, 20, 10, 5), (7, 9, 14, 27)])
def test_linear_image_is_reproduced_away_from_the_border(H, W, oh, ow):
    """Bilinear interpolation is exact for a + b*x + c*y wherever both taps are inside the image."""
    y, x = np.mgrid[0:H, 0:W].astype(np.float64)
    img = (3.0 + 2.0 * x - 1.5 * y)[..., None]
    out = P.resize_bilinear(img, oh, ow)[..., 0]
    sy = (np.arange(oh) + 0.5) * H / oh - 0.5
    sx = (np.arange(ow) + 0.5) * W / ow - 0.5
    inside = (sy[:, None] >= 0) & (sy[:, None] <= H - 1) & (sx[None, :] >= 0) & (sx[None, :] <= W - 1)
    want = 3.0 + 2.0 * sx[None, :] - 1.5 * sy[:, None]
    assert inside.sum() > 0
    np.testing.assert_allclose(out[inside], want[inside], rtol=0, atol=1e-10)
    # outside, the coordinate is clamped to the nearest pixel centre
    want_c = 3.0 + 2.0 * np.clip(sx, 0, W - 1)[None, :] - 1.5 * np.clip(sy, 0, H - 1)[:, None]
    np.testing.assert_allclose(out, want_c, rtol=0, atol=1e-10)


@pytest.mark.parametrize("H,W,oh,ow", [(11, 7, 22, 14), (37, 53, 16, 16), (10, 10, 25, 15), (64, 48, 56, 112)])
def test_resize_matches_torch_interpolate(H, W, oh, ow):
    img = gen.make_image_u8(H, W, 3, seed=H * 100 + W)
    t = torch.from_numpy(img.astype(np.float64)).permute(2, 0, 1)[None]
    want = F.interpolate(t, size=(oh, ow), mode="bilinear", align_corners=False, antialias=False)[0].permute(1, 2, 0).numpy()
    np.testing.assert_allclose(P.resize_bilinear(img, oh, ow), want, rtol=0, atol=1e-9)


def test_normalize_closed_form():
    img = np.array([[[0, 255, 51]]], dtype=np.uint8)
    got = P.normalize(img, MEAN, STD)
    want = [(0.0 - 0.48) / 0.27, (1.0 - 0.45) / 0.26, (0.2 - 0.41) / 0.28]
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-15)


def test_tile_order_and_layout_by_brute_force():
    S, rows, cols = 4, 2, 3
    img = gen.make_image_u8(rows * S, cols * S, 3, seed=5)        # same size as the tiled canvas: resize is the identity
    tiles = P.preprocess_tiles(img, S, rows, cols, True, MEAN, STD)
    assert tiles.shape == (rows * cols + 1, 3, S, S)
    for ty in range(rows):
        for tx in range(cols):
            for c in range(3):
                for y in range(S):
                    for x in range(S):
                        want = (img[ty * S + y, tx * S + x, c] / 255.0 - MEAN[c]) / STD[c]
                        assert abs(tiles[ty * cols + tx, c, y, x] - want) < 1e-12
    thumb = P.normalize(P.resize_bilinear(img, S, S), MEAN, STD).transpose(2, 0, 1)
    np.testing.assert_array_equal(tiles[-1], thumb)
    assert P.preprocess_tiles(img, S, rows, cols, False, MEAN, STD).shape[0] == rows * cols


def test_argument_validation():
    with pytest.raises(ValueError):
        P.preprocess_tiles(np.zeros((4, 4, 3), dtype=np.float32), 4, 1, 1, False, MEAN, STD)
    with pytest.raises(ValueError):
        P.preprocess_tiles(np.zeros((4, 4, 3), dtype=np.uint8), 4, 0, 1, False, MEAN, STD)
