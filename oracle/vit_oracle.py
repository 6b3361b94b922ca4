"""CPU oracle for the packed ViT image encoder.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module; the product path (the HIP library and its Python binding) never does,
and this module imports nothing from the product.

What it computes.  The paper (Sec. 2, "Image Encoding") says the image encoder
takes preprocessed fixed-size tiles and emits image tokens, using the vision
transformer architecture it cites, and (Sec. 3.1, compute characteristics;
Sec. 1) that images of a request never attend to each other.  Packing many
requests' images into one batch is therefore a pure re-layout, and the result has
a plain definition: the textbook pre-LayerNorm ViT forward, evaluated tile by
tile, image by image.  This file is that definition written out with numpy,
in float64 by default (float32 on request), with `@` (matmul) as the only
library primitive; no blocking, fusion or batching across images.

Readings taken where the paper is silent (it gives no ViT equations):
  * patch grid g = floor(S/p); trailing pixels ignored (the only reading that gives
    Table 1's 729 tokens for 384-px tiles with patch 14);
  * patch vector order (c, py, px), i.e. a stride-p convolution kernel flattened;
  * learned CLS row first (if present), learned position table added to every row;
  * block: x += Wo.attn(LN1(x)); x += W2.gelu(W1.LN2(x)); biases everywhere;
  * LN with biased variance; softmax with max subtraction; exact erf GELU;
  * local layer: keys = the tile's own tokens; global layer: keys = all tokens of
    all tiles of the same image in tile order (Table 1: 4 x 1601 = 6404);
  * final LN (optional) then 0/1/2-layer projector with GELU between layers, applied
    to every token; all tokens are output in input tile order;
  * token down-sampling (Table 1 lists 448-px tiles with 256 tokens each, a quarter of the
    32 x 32 patch grid; the paper does not say how): after the final LN the CLS row is
    dropped and every m x m block of neighbouring patch tokens becomes one token whose
    channels are the block's tokens one after the other, rows of the block first; the
    projector then takes m*m*D inputs.

Pins (tests/test_oracle_*.py): Table 1 token counts; patch matmul == brute-force
strided convolution; softmax/LN/GELU closed forms; zero-block identity; single-tile
global == local; bitwise packing invariance; float32 vs float64; and an independent
composition of PyTorch CPU functional ops (conv2d, layer_norm,
scaled_dot_product_attention, gelu, linear) in float64.
Parity with any released, trained encoder is unpinned and not claimed.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf


# --------------------------------------------------------------------------- weights
def unpack_weights(cfg: dict, flat: np.ndarray, dtype=np.float64) -> dict:
    """Split the flat fp32 weight buffer into named arrays (documented interchange order)."""
    D, M = cfg["hidden"], cfg["mlp"]
    p, C = cfg["patch_size"], cfg["channels"]
    g = cfg["image_size"] // p
    T = g * g + (1 if cfg["has_cls"] else 0)
    pos = 0

    def take(*shape):
        nonlocal pos
        n = int(np.prod(shape))
        a = np.asarray(flat[pos:pos + n], dtype=dtype).reshape(shape)
        pos += n
        return a

    w = {"patch_w": take(D, C * p * p), "patch_b": take(D)}
    if cfg["has_cls"]:
        w["cls"] = take(D)
    w["pos"] = take(T, D)
    w["layers"] = []
    for _ in range(cfg["layers_local"] + cfg["layers_global"]):
        w["layers"].append({
            "ln1_g": take(D), "ln1_b": take(D),
            "wqkv": take(3 * D, D), "bqkv": take(3 * D),
            "wo": take(D, D), "bo": take(D),
            "ln2_g": take(D), "ln2_b": take(D),
            "w1": take(M, D), "b1": take(M),
            "w2": take(D, M), "b2": take(D),
        })
    if cfg["final_ln"]:
        w["lnf_g"], w["lnf_b"] = take(D), take(D)
    w["proj"] = []
    d_in = D * max(cfg.get("token_merge", 1), 1) ** 2
    for i in range(cfg["proj_layers"]):
        d_out = cfg["proj_dims"][i]
        w["proj"].append((take(d_out, d_in), take(d_out)))
        d_in = d_out
    if pos != flat.size:
        raise ValueError(f"weight buffer has {flat.size} values, config needs {pos}")
    return w


# --------------------------------------------------------------------------- primitive ops
def tokens_per_tile(cfg: dict) -> int:
    """g^2 patches (+1 CLS); g = floor(S/p).  Table 1: 560/14 -> 1600+1, 384/14 -> 27^2 = 729."""
    g = cfg["image_size"] // cfg["patch_size"]
    return g * g + (1 if cfg["has_cls"] else 0)


def out_tokens_per_tile(cfg: dict) -> int:
    """Tokens a tile hands on: all T, or (g/m)^2 after m x m down-sampling.  Table 1: 448/14 = 32,
    m = 2 -> 16^2 = 256 tokens per tile, 5 tiles -> 1280 per image."""
    m = cfg.get("token_merge", 1)
    if m <= 1:
        return tokens_per_tile(cfg)
    g = cfg["image_size"] // cfg["patch_size"]
    if g % m:
        raise ValueError("the patch grid must be a multiple of token_merge")
    return (g // m) ** 2


def merge_tokens(x: np.ndarray, cfg: dict) -> np.ndarray:
    """Token down-sampling of ONE tile: x [T, D] -> [(g/m)^2, m*m*D].

    Output token (Y, X) is the concatenation of patch tokens (m*Y + dy, m*X + dx) for dy = 0..m-1
    (outer), dx = 0..m-1 (inner); patch (y, x) is row cls + y*g + x of x.  The CLS row is dropped."""
    m = cfg["token_merge"]
    g = cfg["image_size"] // cfg["patch_size"]
    cls = 1 if cfg["has_cls"] else 0
    D = x.shape[1]
    gm = g // m
    out = np.empty((gm * gm, m * m * D), dtype=x.dtype)
    for Y in range(gm):
        for X in range(gm):
            for dy in range(m):
                for dx in range(m):
                    q = dy * m + dx
                    out[Y * gm + X, q * D:(q + 1) * D] = x[cls + (m * Y + dy) * g + (m * X + dx)]
    return out


def linear(x: np.ndarray, w: np.ndarray, b: np.ndarray) -> np.ndarray:
    """y[t, j] = sum_k x[t, k] * w[j, k] + b[j]  (weights stored [out, in])."""
    return x @ w.T + b


def layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """Per row: (x - mean) / sqrt(biased_var + eps) * gamma + beta."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + x.dtype.type(eps)) * gamma + beta


def gelu(z: np.ndarray) -> np.ndarray:
    """Exact GELU: z/2 * (1 + erf(z / sqrt 2))."""
    return (0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))).astype(z.dtype)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Row-wise softmax with the row maximum subtracted first."""
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_segment(q: np.ndarray, k: np.ndarray, v: np.ndarray, heads: int) -> np.ndarray:
    """Multi-head self-attention inside one segment.

    q, k, v: [n, D] with head h occupying columns h*dh .. (h+1)*dh.  For each head,
    A = softmax_rows(q_h k_h^T / sqrt(dh)) over the n keys of the segment, out_h = A v_h.
    """
    n, D = q.shape
    dh = D // heads
    out = np.empty_like(q)
    scale = q.dtype.type(1.0 / math.sqrt(dh))
    for h in range(heads):
        c = slice(h * dh, (h + 1) * dh)
        a = softmax_rows((q[:, c] @ k[:, c].T) * scale)
        out[:, c] = a @ v[:, c]
    return out


def extract_patches(tile: np.ndarray, p: int) -> np.ndarray:
    """[C, S, S] -> [g*g, C*p*p]; patch (gy, gx) row-major, vector index c*p*p + py*p + px."""
    C, S, _ = tile.shape
    g = S // p
    v = tile[:, :g * p, :g * p].reshape(C, g, p, g, p)      # c, gy, py, gx, px
    return v.transpose(1, 3, 0, 2, 4).reshape(g * g, C * p * p)


def patch_embed(tile: np.ndarray, w: dict, cfg: dict) -> np.ndarray:
    """Tile -> token matrix [T, D]: patch projection + bias, CLS row first, + position table."""
    e = linear(extract_patches(tile, cfg["patch_size"]), w["patch_w"], w["patch_b"])
    if cfg["has_cls"]:
        e = np.concatenate([w["cls"][None, :], e], axis=0)
    return e + w["pos"]


def block(x: np.ndarray, lw: dict, cfg: dict, segments) -> np.ndarray:
    """One pre-LN transformer block over x [n, D]; `segments` lists (start, stop) key ranges."""
    D = cfg["hidden"]
    h = layer_norm(x, lw["ln1_g"], lw["ln1_b"], cfg["ln_eps"])
    qkv = linear(h, lw["wqkv"], lw["bqkv"])
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    o = np.empty_like(x)
    for a, b in segments:
        o[a:b] = attention_segment(q[a:b], k[a:b], v[a:b], cfg["heads"])
    x = x + linear(o, lw["wo"], lw["bo"])
    h = layer_norm(x, lw["ln2_g"], lw["ln2_b"], cfg["ln_eps"])
    x = x + linear(gelu(linear(h, lw["w1"], lw["b1"])), lw["w2"], lw["b2"])
    return x


def encode_image(tiles: np.ndarray, w: dict, cfg: dict) -> np.ndarray:
    """All tiles of ONE image [n, C, S, S] -> [n*T_out, out_dim]."""
    n = tiles.shape[0]
    T = tokens_per_tile(cfg)
    x = np.concatenate([patch_embed(tiles[i], w, cfg) for i in range(n)], axis=0)
    local = [(i * T, (i + 1) * T) for i in range(n)]
    whole = [(0, n * T)]
    for l, lw in enumerate(w["layers"]):
        x = block(x, lw, cfg, local if l < cfg["layers_local"] else whole)
    if cfg["final_ln"]:
        x = layer_norm(x, w["lnf_g"], w["lnf_b"], cfg["ln_eps"])
    if cfg.get("token_merge", 1) > 1:
        x = np.concatenate([merge_tokens(x[i * T:(i + 1) * T], cfg) for i in range(n)], axis=0)
    for i, (pw, pb) in enumerate(w["proj"]):
        if i > 0:
            x = gelu(x)
        x = linear(x, pw, pb)
    return x


# --------------------------------------------------------------------------- packed entry point
def request_token_offsets(cfg: dict, images_per_request, tile_offsets) -> np.ndarray:
    """Prefix sums: first output token row of each request (length n_requests + 1)."""
    T = out_tokens_per_tile(cfg)
    ipr = np.asarray(images_per_request, dtype=np.int64)
    to = np.asarray(tile_offsets, dtype=np.int64)
    img_end = np.concatenate([[0], np.cumsum(ipr)])
    return to[img_end] * T


def vit_oracle_encode(cfg: dict, weights, pixels: np.ndarray, images_per_request, tile_offsets,
                      dtype=np.float64, images=None):
    """Encode a packed batch.  Returns (tokens [n_tiles*T_out, out_dim], request_token_offsets).

    `weights` is the flat buffer or an already unpacked dict.  `images`, if given, lists
    the image indices to encode; rows of other images are left as NaN (each image's
    tokens depend on its own tiles only, so a sample of whole images is exact).
    """
    ipr = np.asarray(images_per_request, dtype=np.int64)
    to = np.asarray(tile_offsets, dtype=np.int64)
    if (ipr < 0).any():
        raise ValueError("images_per_request must be non-negative")
    n_images = int(ipr.sum())
    if to.shape[0] != n_images + 1 or to[0] != 0 or (np.diff(to) < 1).any():
        raise ValueError("tile_offsets must be a prefix sum with at least one tile per image")
    if pixels.shape[0] != to[-1]:
        raise ValueError("pixels hold a different number of tiles than tile_offsets")
    w = weights if isinstance(weights, dict) else unpack_weights(cfg, weights, dtype)
    T = out_tokens_per_tile(cfg)
    out_dim = (cfg["proj_dims"][cfg["proj_layers"] - 1] if cfg["proj_layers"]
               else cfg["hidden"] * max(cfg.get("token_merge", 1), 1) ** 2)
    out = np.full((int(to[-1]) * T, out_dim), np.nan, dtype=dtype)
    for i in (range(n_images) if images is None else images):
        a, b = int(to[i]), int(to[i + 1])
        out[a * T:b * T] = encode_image(np.asarray(pixels[a:b], dtype=dtype), w, cfg)
    return out, request_token_offsets(cfg, ipr, to)
