"""Second opinion for the oracle: the same network composed from PyTorch CPU library ops in float64.

conv2d (stride = kernel), layer_norm, scaled_dot_product_attention, gelu and linear are
library routines with their own implementations; none of the oracle's code is reused.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import gen
from oracle import vit_oracle as O


def torch_encode_image(cfg, flat, tiles):
    """tiles [n, C, S, S] of one image -> [n*T_out, out_dim] float64."""
    f = torch.from_numpy(np.asarray(flat, dtype=np.float64))
    pos = 0

    def take(*shape):
        nonlocal pos
        n = int(np.prod(shape))
        t = f[pos:pos + n].reshape(shape)
        pos += n
        return t

    D, M, H = cfg["hidden"], cfg["mlp"], cfg["heads"]
    p, C, S = cfg["patch_size"], cfg["channels"], cfg["image_size"]
    g = S // p
    T = g * g + cfg["has_cls"]
    n = tiles.shape[0]
    x = torch.from_numpy(np.asarray(tiles, dtype=np.float64))
    conv_w, conv_b = take(D, C, p, p), take(D)
    x = F.conv2d(x, conv_w, conv_b, stride=p)                 # [n, D, g, g]; floor(S/p) grid
    x = x.flatten(2).transpose(1, 2)                          # [n, g*g, D]
    if cfg["has_cls"]:
        cls = take(D)
        x = torch.cat([cls.expand(n, 1, D), x], dim=1)
    x = x + take(T, D)
    L = cfg["layers_local"] + cfg["layers_global"]
    for l in range(L):
        g1, b1 = take(D), take(D)
        wqkv, bqkv, wo, bo = take(3 * D, D), take(3 * D), take(D, D), take(D)
        g2, b2 = take(D), take(D)
        w1, bb1, w2, bb2 = take(M, D), take(M), take(D, M), take(D)
        if l >= cfg["layers_local"]:
            x = x.reshape(1, n * T, D)                        # all tiles of the image form one sequence
        B, N, _ = x.shape
        h = F.layer_norm(x, (D,), g1, b1, cfg["ln_eps"])
        q, k, v = F.linear(h, wqkv, bqkv).reshape(B, N, 3, H, D // H).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v)           # default scale 1/sqrt(dh)
        x = x + F.linear(a.transpose(1, 2).reshape(B, N, D), wo, bo)
        h = F.layer_norm(x, (D,), g2, b2, cfg["ln_eps"])
        x = x + F.linear(F.gelu(F.linear(h, w1, bb1)), w2, bb2)
    x = x.reshape(n * T, D)
    if cfg["final_ln"]:
        x = F.layer_norm(x, (D,), take(D), take(D), cfg["ln_eps"])
    d_in = D
    m = cfg["token_merge"]
    if m > 1:
        # library routine: pixel_unshuffle turns [*, D, g, g] into [*, D*m*m, g/m, g/m] with channel
        # index c*m*m + dy*m + dx; the encoder's channel order is (dy, dx, c), hence the permute
        x = x.reshape(n, T, D)[:, cfg["has_cls"]:, :].transpose(1, 2).reshape(n, D, g, g)
        x = F.pixel_unshuffle(x, m)                           # [n, D*m*m, g/m, g/m]
        x = x.reshape(n, D, m * m, (g // m) ** 2).permute(0, 3, 2, 1).reshape(n * (g // m) ** 2, m * m * D)
        d_in = m * m * D
    for i in range(cfg["proj_layers"]):
        d_out = cfg["proj_dims"][i]
        if i > 0:
            x = F.gelu(x)
        x = F.linear(x, take(d_out, d_in), take(d_out))
        d_in = d_out
    assert pos == f.numel()
    return x.numpy()


CASES = [
    ("test_small_fp32", [1, 3, 2]),
    ("test_dh72_bf16", [2, 1]),
    ("test_dh80_bf16", [3, 1]),
    ("test_medium_fp32", [2]),
    ("cfg1_tiny_fp32", [1, 1]),
    ("test_dh96_bf16", [2, 1]),
    ("test_dh128_bf16", [1, 2]),
    ("test_merge_fp32", [2, 1]),
    ("test_merge3_bf16", [1, 2]),
]


@pytest.mark.parametrize("name,tpi", CASES)
def test_oracle_matches_torch_functional(name, tpi):
    cfg = gen.get_config(name)
    flat = gen.make_weights(cfg, seed=0)
    # scale the weights up so attention is far from uniform and GELU far from linear
    flat = gen.round_to_bf16(flat * 4.0) if cfg["dtype"] == "bf16" else flat * 4.0
    to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
    px = gen.make_pixels(cfg, int(to[-1]), seed=1)
    out, _ = O.vit_oracle_encode(cfg, flat, px, [len(tpi)], to)
    T = O.out_tokens_per_tile(cfg)
    for i in range(len(tpi)):
        want = torch_encode_image(cfg, flat, px[to[i]:to[i + 1]])
        got = out[to[i] * T:to[i + 1] * T]
        assert got.shape == want.shape
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)
