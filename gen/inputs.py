"""Seeded weights, pixels and request structure (inputs only, no encoder arithmetic).

Stand-ins for the paper's workloads, which are not available here: its production
trace (images per request: heavy-tailed, Sec. 3.3) and its image dataset.  Only
the published shape of those workloads is used: heavy-tailed image counts,
fixed-size tiles per model (Table 1).
"""
from __future__ import annotations

import numpy as np

from .configs import get_config, tokens_per_tile, weight_layout

# Config 3: images per request, clip(rint(LogNormal(0, 1.8)), 1, 32) drawn once; this list is the contract.
CFG3_IMAGES_PER_REQUEST = [
    1, 1, 3, 1, 1, 2, 10, 5, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 2, 7, 1, 12, 1, 2, 5, 1, 1, 1, 1, 1, 1, 1,
    1, 3, 1, 2, 1, 1, 4, 15, 1, 15, 11, 4, 2, 1, 14, 32, 26, 11, 2, 1, 1, 3, 1, 2, 2, 4, 1, 1, 1, 1, 23, 1,
]
# Config 4: tiles per image = U{1..6} dynamic tiles + 1 thumbnail; drawn once; this list is the contract.
CFG4_TILES_PER_IMAGE = [
    7, 5, 5, 3, 3, 2, 2, 2, 3, 6, 5, 7, 5, 5, 7, 6, 5, 5, 5, 7, 3, 6, 6, 2, 4, 7, 5, 2, 6, 6, 7, 3,
    2, 7, 2, 5, 2, 3, 4, 4, 4, 2, 2, 2, 2, 6, 5, 5, 3, 5, 6, 4, 4, 7, 6, 7, 4, 6, 7, 5, 7, 6, 6, 4,
    7, 2, 5, 6, 7, 5, 4, 3, 4, 4, 6, 7, 2, 7, 5, 4, 6, 5, 3, 3, 6, 5, 5, 4, 6, 4, 3, 7, 3, 3, 6, 5,
    2, 2, 4, 6, 4, 6, 3, 3, 6, 7, 2, 2, 6, 4, 5, 2, 7, 4, 7, 6, 6, 3, 6, 2, 5, 4, 7, 3, 7, 2, 5, 5,
]
assert sum(CFG3_IMAGES_PER_REQUEST) == 260 and len(CFG3_IMAGES_PER_REQUEST) == 64
assert sum(CFG4_TILES_PER_IMAGE) == 591 and len(CFG4_TILES_PER_IMAGE) == 128


def _round_to_bf16_inplace(a: np.ndarray) -> np.ndarray:
    u = a.reshape(-1).view(np.uint32)  # finite inputs only: the add below cannot wrap
    step = 1 << 26                      # in pieces, so the temporaries stay small
    for i in range(0, u.size, step):
        v = u[i:i + step]
        lsb = (v >> np.uint32(16)) & np.uint32(1)
        v += np.uint32(0x7FFF)
        v += lsb
        v &= np.uint32(0xFFFF0000)
    return a


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Return fp32 values that are exactly representable in bfloat16 (round-to-nearest-even)."""
    return _round_to_bf16_inplace(np.array(a, dtype=np.float32, order="C", copy=True))


def make_weights(cfg: dict, seed: int = 0) -> np.ndarray:
    """Flat fp32 weight buffer in ``weight_layout`` order.

    Every matrix, embedding, CLS vector and bias ~ N(0, 0.02^2); LayerNorm gains
    ~ 1 + N(0, 0.02^2).  For bf16 configs every value is rounded once to a
    bf16-representable fp32 so both sides consume identical weights.
    """
    rng = np.random.default_rng(seed)
    layout = weight_layout(cfg)
    sizes = [int(np.prod(shape)) for _, shape in layout]
    flat = np.empty(sum(sizes), dtype=np.float32)  # filled in place: the largest preset has 5.65 G values
    pos = 0
    for (name, _), n in zip(layout, sizes):
        w = flat[pos:pos + n]
        rng.standard_normal(out=w, dtype=np.float32)
        w *= np.float32(0.02)
        if name.endswith(("ln1_g", "ln2_g", "lnf_g")):
            w += np.float32(1.0)
        pos += n
    if cfg["dtype"] == "bf16":
        flat = _round_to_bf16_inplace(flat)
    return flat


def make_pixels(cfg: dict, n_tiles: int, seed: int = 1) -> np.ndarray:
    """[n_tiles, C, S, S] fp32 pixels ~ U[-1, 1) (already-normalised tiles)."""
    rng = np.random.default_rng(seed)
    S, C = cfg["image_size"], cfg["channels"]
    px = rng.random((n_tiles, C, S, S), dtype=np.float32)
    px *= np.float32(2.0)
    px -= np.float32(1.0)
    return px


def make_image_u8(height: int, width: int, channels: int = 3, seed: int = 0) -> np.ndarray:
    """[H, W, C] uint8 raw image: smooth low-frequency content plus noise, so that interpolation between
    neighbouring pixels is neither trivial nor pure noise."""
    rng = np.random.default_rng(seed)
    y, x = np.mgrid[0:height, 0:width].astype(np.float32)
    img = np.empty((height, width, channels), dtype=np.float32)
    for c in range(channels):
        fy, fx, ph = rng.uniform(0.01, 0.2), rng.uniform(0.01, 0.2), rng.uniform(0, 6.28)
        img[..., c] = 127.5 + 90.0 * np.sin(fy * y + fx * x + ph)
    img += rng.normal(0.0, 20.0, img.shape).astype(np.float32)
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


def make_workload(name: str):
    """Return (cfg, images_per_request, tile_offsets) for a named benchmark workload.

    tile_offsets is the prefix sum of tiles per image, length n_images + 1.
    """
    if name == "cfg1":
        cfg, ipr, tpi = get_config("cfg1_tiny_fp32"), [1] * 4, [1] * 4
    elif name == "cfg2":
        cfg, ipr, tpi = get_config("cfg2_vitl14_336"), [1] * 8, [1] * 8
    elif name == "cfg3":
        cfg, ipr = get_config("cfg2_vitl14_336"), list(CFG3_IMAGES_PER_REQUEST)
        tpi = [1] * sum(ipr)
    elif name == "cfg4":
        cfg, ipr, tpi = get_config("cfg4_siglip_384"), [1] * 128, list(CFG4_TILES_PER_IMAGE)
    elif name == "cfg5":
        cfg, ipr, tpi = get_config("cfg5_vith14_560"), [1] * 32, [4] * 32
    elif name == "cfg6":
        # second workload: seven images of five 448-px tiles (Table 1: 5 x 256 tokens for an 896-px image)
        # and one single-tile image, small enough for the oracle to encode at full width and depth
        cfg, ipr, tpi = get_config("cfg6_6b_448"), [1] * 8, [5] * 7 + [1]
    else:
        raise KeyError(name)
    tile_offsets = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
    return cfg, np.asarray(ipr, dtype=np.int32), tile_offsets


__all__ = [
    "CFG3_IMAGES_PER_REQUEST", "CFG4_TILES_PER_IMAGE", "round_to_bf16", "make_weights",
    "make_pixels", "make_workload", "make_image_u8", "make_arrivals", "tokens_per_tile",
]


def make_arrivals(n_requests: int, mean_interarrival_ms: float, seed: int = 0, tiles_per_image: int = 1,
                  max_images: int = 32):
    """Seeded request stream for the routing experiments: Poisson arrivals, images per request drawn
    from the same heavy-tailed recipe as the ragged batch (log-normal(0, 1.8), rounded, clipped to
    [1, max_images]: median 1, a few requests with tens of images).  Returns a list of
    (arrival time in ms, [tiles of every image])."""
    rng = np.random.default_rng(seed)
    t = 0.0
    out = []
    for _ in range(n_requests):
        t += float(rng.exponential(mean_interarrival_ms))
        n = int(np.clip(np.rint(rng.lognormal(0.0, 1.8)), 1, max_images))
        out.append((t, [tiles_per_image] * n))
    return out
