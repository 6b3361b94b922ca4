"""The oracle's pins must notice a plausible mistake anywhere in it.

Each case plants one mistake in the ORACLE (on the CPU, through monkeypatching one of its functions), runs
the pin that compares it with the independent composition of PyTorch library ops, and requires the
disagreement to exceed that pin's tolerance by orders of magnitude.  With no mistake planted the same
comparison agrees to 1e-9 (`test_oracle_torch.py`).
"""
import math

import numpy as np
import pytest

import gen
from oracle import vit_oracle as O
from test_oracle_torch import torch_encode_image

PIN_TOLERANCE = 1e-9   # the relative tolerance of test_oracle_matches_torch_functional
NOTICED = 1e-4         # a planted mistake must move the comparison at least this far (observed: 1.3e-3 ... 1.4)


def _disagreement(name="test_medium_fp32", tpi=(2, 1)):
    """Largest relative difference between the oracle and the PyTorch composition over the images."""
    cfg = gen.get_config(name)
    flat = gen.make_weights(cfg, seed=0) * 4.0
    to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
    px = gen.make_pixels(cfg, int(to[-1]), seed=1)
    out, _ = O.vit_oracle_encode(cfg, flat, px, [len(tpi)], to)
    T = O.out_tokens_per_tile(cfg)
    worst = 0.0
    for i in range(len(tpi)):
        want = torch_encode_image(cfg, flat, px[to[i]:to[i + 1]])
        got = out[to[i] * T:to[i + 1] * T]
        worst = max(worst, float(np.abs(got - want).max() / np.abs(want).max()))
    return worst


def test_without_a_mistake_the_pin_agrees():
    assert _disagreement() < PIN_TOLERANCE
    assert _disagreement("test_merge_fp32", (2, 1)) < PIN_TOLERANCE


def _tanh_gelu(z):
    return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))


def _unbiased_layer_norm(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(x.var(axis=-1, ddof=1, keepdims=True) + eps) * gamma + beta


def _softmax_without_max_and_wrong_axis(s):
    e = np.exp(s - s.max())
    return e / e.sum(axis=0, keepdims=True)      # normalises over queries instead of keys


MISTAKES = {
    "tanh form of GELU": ("gelu", lambda orig: _tanh_gelu),
    "GELU without the 1/2": ("gelu", lambda orig: (lambda z: 2.0 * orig(z))),
    "unbiased variance in LayerNorm": ("layer_norm", lambda orig: _unbiased_layer_norm),
    "LayerNorm eps ten times too large": ("layer_norm", lambda orig: (lambda x, g, b, eps: orig(x, g, b, eps * 10.0))),
    "LayerNorm without beta": ("layer_norm", lambda orig: (lambda x, g, b, eps: orig(x, g, np.zeros_like(b), eps))),
    "linear layer without its bias": ("linear", lambda orig: (lambda x, w, b: x @ w.T)),
    "square weight used untransposed": ("linear", lambda orig: (lambda x, w, b: (x @ w if w.shape[0] == w.shape[1] else x @ w.T) + b)),
    "softmax over the wrong axis": ("softmax_rows", lambda orig: _softmax_without_max_and_wrong_axis),
    "logits not scaled by 1/sqrt(dh)": ("softmax_rows", lambda orig: (lambda s: orig(s * 8.0))),   # dh = 64
    "heads not separated (one head over D)": ("attention_segment", lambda orig: (lambda q, k, v, heads: orig(q, k, v, 1))),
    "keys and queries swapped": ("attention_segment", lambda orig: (lambda q, k, v, heads: orig(k, q, v, heads))),
    "patch vector in (py, px, c) order": ("extract_patches", lambda orig: (
        lambda tile, p: orig(tile, p).reshape(-1, tile.shape[0], p * p).transpose(0, 2, 1).reshape(-1, tile.shape[0] * p * p))),
    "position table not added": ("patch_embed", lambda orig: (lambda tile, w, cfg: orig(tile, w, cfg) - w["pos"])),
}


@pytest.mark.parametrize("what", sorted(MISTAKES))
def test_a_planted_mistake_is_noticed(what, monkeypatch):
    attr, make = MISTAKES[what]
    monkeypatch.setattr(O, attr, make(getattr(O, attr)))
    d = _disagreement()
    assert d > NOTICED, (what, d)


def test_global_layers_and_token_order_mistakes_are_noticed(monkeypatch):
    # a global layer that attends inside tiles only: plant it by making every layer local
    orig = O.encode_image

    def all_local(tiles, w, cfg):
        return orig(tiles, w, dict(cfg, layers_local=cfg["layers_local"] + cfg["layers_global"], layers_global=0))

    monkeypatch.setattr(O, "encode_image", all_local)
    assert _disagreement() > NOTICED
    monkeypatch.setattr(O, "encode_image", orig)
    # token down-sampling with the block's tokens in (dx, dy) order instead of (dy, dx)
    merge = O.merge_tokens

    def transposed_blocks(x, cfg):
        m, D = cfg["token_merge"], cfg["hidden"]
        y = merge(x, cfg)
        return y.reshape(y.shape[0], m, m, D).transpose(0, 2, 1, 3).reshape(y.shape[0], m * m * D)

    monkeypatch.setattr(O, "merge_tokens", transposed_blocks)
    assert _disagreement("test_merge_fp32", (2, 1)) > NOTICED
