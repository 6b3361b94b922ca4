"""Pins for the CPU oracle against facts fixed by the paper and by mathematics (no GPU)."""
import math
import os

import numpy as np
import pytest

import gen
from oracle import vit_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def tiny_cfg(**kw):
    cfg = gen.get_config("test_small_fp32")
    cfg.update(kw)
    return cfg


# ------------------------------------------------------------------ paper-printed values
def test_table1_token_counts():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "table1_token_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for S, p, cls, m, T, n, total in (map(int, r) for r in rows):
        cfg = tiny_cfg(image_size=S, patch_size=p, has_cls=cls, token_merge=m)
        assert O.out_tokens_per_tile(cfg) == T
        assert n * O.out_tokens_per_tile(cfg) == total
        assert gen.out_tokens_per_tile(cfg) == T
        if m == 1:
            assert O.tokens_per_tile(cfg) == T and gen.tokens_per_tile(cfg) == T


def test_config_shapes():
    assert O.tokens_per_tile(gen.get_config("cfg1_tiny_fp32")) == 197
    assert O.tokens_per_tile(gen.get_config("cfg2_vitl14_336")) == 577
    assert O.tokens_per_tile(gen.get_config("cfg4_siglip_384")) == 729
    assert O.tokens_per_tile(gen.get_config("cfg5_vith14_560")) == 1601
    cfg6 = gen.get_config("cfg6_6b_448")
    assert O.tokens_per_tile(cfg6) == 1025 and O.out_tokens_per_tile(cfg6) == 256


# ------------------------------------------------------------------ token down-sampling
def test_token_merge_by_hand():
    """2 x 2 grid, D = 2, CLS: the four patch tokens end up side by side in (row, column) order."""
    cfg = tiny_cfg(image_size=4, patch_size=2, has_cls=1, token_merge=2)
    x = np.array([[9., 9.], [1., 2.], [3., 4.], [5., 6.], [7., 8.]])
    np.testing.assert_array_equal(O.merge_tokens(x, cfg), [[1., 2., 3., 4., 5., 6., 7., 8.]])
    # 4 x 4 grid, D = 1, no CLS, value = 10*y + x: token (Y, X) holds its block row by row
    cfg = tiny_cfg(image_size=8, patch_size=2, has_cls=0, token_merge=2)
    x = np.array([[10. * y + xx] for y in range(4) for xx in range(4)])
    np.testing.assert_array_equal(O.merge_tokens(x, cfg),
                                  [[0, 1, 10, 11], [2, 3, 12, 13], [20, 21, 30, 31], [22, 23, 32, 33]])


@pytest.mark.parametrize("g,m,cls,D", [(4, 2, 1, 3), (6, 3, 0, 2), (6, 2, 1, 5), (8, 4, 0, 1)])
def test_token_merge_is_a_reshape_transpose_and_a_permutation(g, m, cls, D):
    cfg = tiny_cfg(image_size=g * 2, patch_size=2, has_cls=cls, token_merge=m)
    x = np.arange((g * g + cls) * D, dtype=np.float64).reshape(g * g + cls, D) + 1.0
    got = O.merge_tokens(x, cfg)
    gm = g // m
    # the same re-layout as one reshape / transpose of the patch grid
    want = x[cls:].reshape(gm, m, gm, m, D).transpose(0, 2, 1, 3, 4).reshape(gm * gm, m * m * D)
    np.testing.assert_array_equal(got, want)
    # every patch value exactly once, the CLS values (if any) not at all
    assert sorted(got.ravel().tolist()) == sorted(x[cls:].ravel().tolist())
    assert O.out_tokens_per_tile(cfg) == gm * gm


def test_token_merge_sits_between_final_ln_and_projector():
    """Encoder with down-sampling == down-sampling applied by hand to the encoder without it (no
    projector), and == projector applied by hand to that (1-layer projector)."""
    base = gen.get_config("test_merge_fp32")
    base.update(proj_layers=0, proj_dims=())
    plain = dict(base, token_merge=1)
    flat = gen.make_weights(plain, seed=3)
    px = gen.make_pixels(plain, 3, seed=4)
    T = O.tokens_per_tile(plain)
    full, _ = O.vit_oracle_encode(plain, flat, px, [2], [0, 1, 3])
    merged, rto = O.vit_oracle_encode(base, flat, px, [2], [0, 1, 3])
    want = np.concatenate([O.merge_tokens(full[t * T:(t + 1) * T], base) for t in range(3)])
    np.testing.assert_array_equal(merged, want)
    assert rto.tolist() == [0, 3 * O.out_tokens_per_tile(base)]
    withp = dict(base, proj_layers=1, proj_dims=(24,))
    rng = np.random.default_rng(5)
    pw, pb = rng.standard_normal((24, 4 * base["hidden"])), rng.standard_normal(24)
    flat_p = np.concatenate([flat, pw.ravel(), pb]).astype(np.float64)
    got, _ = O.vit_oracle_encode(withp, flat_p, px, [2], [0, 1, 3])
    np.testing.assert_allclose(got, want @ pw.T + pb, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ patchify
def test_patch_matmul_equals_direct_convolution():
    """Brute force: a stride-p valid convolution written as nested loops."""
    rng = np.random.default_rng(5)
    C, S, p, D = 3, 11, 3, 4          # 11 = 3*3 + 2: trailing pixels must be ignored
    g = S // p
    tile = rng.standard_normal((C, S, S))
    kern = rng.standard_normal((D, C, p, p))
    bias = rng.standard_normal(D)
    direct = np.zeros((g, g, D))
    for gy in range(g):
        for gx in range(g):
            for j in range(D):
                acc = 0.0
                for c in range(C):
                    for py in range(p):
                        for px in range(p):
                            acc += kern[j, c, py, px] * tile[c, gy * p + py, gx * p + px]
                direct[gy, gx, j] = acc + bias[j]
    got = O.linear(O.extract_patches(tile, p), kern.reshape(D, -1), bias)
    assert got.shape == (g * g, D)
    np.testing.assert_allclose(got, direct.reshape(g * g, D), rtol=0, atol=1e-12)


def test_patch_embed_cls_and_position():
    cfg = tiny_cfg()
    w = O.unpack_weights(cfg, gen.make_weights(cfg, seed=3))
    tile = gen.make_pixels(cfg, 1, seed=4)[0].astype(np.float64)
    x = O.patch_embed(tile, w, cfg)
    T = O.tokens_per_tile(cfg)
    assert x.shape == (T, cfg["hidden"])
    np.testing.assert_allclose(x[0], w["cls"] + w["pos"][0], atol=1e-15)
    # patch (gy=1, gx=2) -> token 1 + 1*g + 2, by hand
    p, g = cfg["patch_size"], cfg["image_size"] // cfg["patch_size"]
    v = tile[:, p:2 * p, 2 * p:3 * p].reshape(-1)
    t = 1 + g + 2
    np.testing.assert_allclose(x[t], w["patch_w"] @ v + w["patch_b"] + w["pos"][t], atol=1e-12)


# ------------------------------------------------------------------ softmax / attention
def test_softmax_rows_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(0)
    s = rng.standard_normal((7, 33)) * 30
    a = O.softmax_rows(s)
    np.testing.assert_allclose(a.sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(O.softmax_rows(s + 1000.0), a, atol=1e-12)
    a32 = O.softmax_rows(s.astype(np.float32))
    np.testing.assert_allclose(a32.sum(-1), 1.0, atol=1e-6)
    # two-key closed form: softmax([a, b]) = [sigmoid(a-b), sigmoid(b-a)]
    np.testing.assert_allclose(O.softmax_rows(np.array([[0.3, -1.1]]))[0, 0], 1 / (1 + math.exp(-1.4)), atol=1e-15)


def test_attention_closed_forms():
    rng = np.random.default_rng(1)
    n, H, dh = 9, 2, 4
    k = rng.standard_normal((n, H * dh))
    v = rng.standard_normal((n, H * dh))
    # q = 0 -> uniform weights -> output is the column mean of V
    out = O.attention_segment(np.zeros((n, H * dh)), k, v, H)
    np.testing.assert_allclose(out, np.broadcast_to(v.mean(0), out.shape), atol=1e-12)
    # a single-token segment returns v
    out = O.attention_segment(k[:1], k[:1], v[:1], H)
    np.testing.assert_allclose(out, v[:1], atol=1e-15)
    # heads do not mix: changing head 1's k/v leaves head 0's output alone
    q = rng.standard_normal((n, H * dh))
    base = O.attention_segment(q, k, v, H)
    k2, v2 = k.copy(), v.copy()
    k2[:, dh:] += 1.0
    v2[:, dh:] -= 2.0
    np.testing.assert_array_equal(O.attention_segment(q, k2, v2, H)[:, :dh], base[:, :dh])


def test_attention_brute_force_with_scale():
    """Loop-level definition incl. the 1/sqrt(dh) logit scale, on a tiny segment."""
    rng = np.random.default_rng(2)
    n, H, dh = 5, 3, 2
    q, k, v = (rng.standard_normal((n, H * dh)) for _ in range(3))
    want = np.zeros((n, H * dh))
    for h in range(H):
        for i in range(n):
            logits = [sum(q[i, h * dh + d] * k[j, h * dh + d] for d in range(dh)) / math.sqrt(dh) for j in range(n)]
            m = max(logits)
            e = [math.exp(l - m) for l in logits]
            z = sum(e)
            for d in range(dh):
                want[i, h * dh + d] = sum(e[j] / z * v[j, h * dh + d] for j in range(n))
    np.testing.assert_allclose(O.attention_segment(q, k, v, H), want, atol=1e-13)


# ------------------------------------------------------------------ LayerNorm / GELU
def test_layer_norm_closed_forms():
    rng = np.random.default_rng(3)
    D, eps = 64, 1e-6
    x = rng.standard_normal((5, D)) * 3 + 2
    one, zero = np.ones(D), np.zeros(D)
    y = O.layer_norm(x, one, zero, eps)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-12)
    var = x.var(-1)                      # biased
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    # unbiased variance would give a different, detectable number
    y_unbiased = (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, ddof=1) + eps)[:, None]
    assert np.abs(y - y_unbiased).max() > 1e-3
    np.testing.assert_allclose(y, (x - x.mean(-1, keepdims=True)) / np.sqrt(var + eps)[:, None], rtol=1e-12)
    # constant row -> beta
    b = rng.standard_normal(D)
    gmm = rng.standard_normal(D)
    np.testing.assert_allclose(O.layer_norm(np.full((1, D), 7.5), gmm, b, eps), b[None], atol=1e-12)
    # scale invariance (up to eps)
    np.testing.assert_allclose(O.layer_norm(10 * x, gmm, b, eps), O.layer_norm(x, gmm, b, eps), atol=1e-6)
    # hand case: x = [1, 3], mean 2, biased var 1 -> [-1, 1]/sqrt(1+eps)
    y = O.layer_norm(np.array([[1.0, 3.0]]), np.array([2.0, 2.0]), np.array([0.5, 0.5]), 0.0)
    np.testing.assert_allclose(y, [[-1.5, 2.5]], atol=1e-15)


def test_gelu_closed_forms_and_table():
    z = np.linspace(-8, 8, 401)
    gz = O.gelu(z)
    assert O.gelu(np.zeros(1))[0] == 0.0
    np.testing.assert_allclose(gz - O.gelu(-z), z, atol=1e-14)           # gelu(z) - gelu(-z) = z
    np.testing.assert_allclose(O.gelu(np.array([6.0, 7.5, 10.0])), [6.0, 7.5, 10.0], rtol=1e-8)
    assert (np.diff(gz[z >= 0]) > 0).all()
    want = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in z])   # libm erf
    np.testing.assert_allclose(gz, want, atol=1e-15)
    # value from the normal CDF: gelu(1) = Phi(1) = 0.8413447460685429...
    np.testing.assert_allclose(O.gelu(np.array([1.0]))[0], 0.8413447460685429, atol=1e-15)
    # the tanh approximation differs by > 1e-4 somewhere: the oracle must be the erf form
    tanh_form = 0.5 * z * (1 + np.tanh(math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)))
    assert np.abs(tanh_form - gz).max() > 1e-4


# ------------------------------------------------------------------ whole network
def _small_inputs(cfg, tiles_per_image, seed=0):
    to = np.concatenate([[0], np.cumsum(tiles_per_image)]).astype(np.int32)
    px = gen.make_pixels(cfg, int(to[-1]), seed=seed + 1)
    return to, px


def test_zero_blocks_are_identity():
    """All block weights zero -> output = LN_f(patch embedding + pos)."""
    cfg = tiny_cfg(proj_layers=0, proj_dims=())
    flat = gen.make_weights(cfg, seed=0)
    w = O.unpack_weights(cfg, flat)
    for lw in w["layers"]:
        for k in ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2"):
            lw[k][...] = 0
    to, px = _small_inputs(cfg, [1, 2])
    out, _ = O.vit_oracle_encode(cfg, w, px, [2], to)
    T = O.tokens_per_tile(cfg)
    for t in range(3):
        want = O.layer_norm(O.patch_embed(px[t].astype(np.float64), w, cfg), w["lnf_g"], w["lnf_b"], cfg["ln_eps"])
        np.testing.assert_allclose(out[t * T:(t + 1) * T], want, atol=1e-13)


def test_single_tile_global_equals_local():
    cfg_g = tiny_cfg(layers_local=1, layers_global=2)
    cfg_l = tiny_cfg(layers_local=3, layers_global=0)
    flat = gen.make_weights(cfg_g, seed=2)
    to, px = _small_inputs(cfg_g, [1, 1, 1])
    a, _ = O.vit_oracle_encode(cfg_g, flat, px, [3], to)
    b, _ = O.vit_oracle_encode(cfg_l, flat, px, [3], to)
    np.testing.assert_array_equal(a, b)


def test_global_layers_mix_tiles_of_one_image_only():
    cfg = tiny_cfg(layers_local=1, layers_global=1)
    flat = gen.make_weights(cfg, seed=2)
    to, px = _small_inputs(cfg, [2, 1])
    T = O.tokens_per_tile(cfg)
    base, _ = O.vit_oracle_encode(cfg, flat, px, [1, 1], to)
    px2 = px.copy()
    px2[1] += 0.25                     # second tile of image 0
    out, _ = O.vit_oracle_encode(cfg, flat, px2, [1, 1], to)
    assert np.abs(out[:T] - base[:T]).max() > 1e-6           # tile 0 sees tile 1 through the global layer
    np.testing.assert_array_equal(out[2 * T:], base[2 * T:])  # image 1 untouched
    cfg_loc = tiny_cfg(layers_local=2, layers_global=0)
    base_l, _ = O.vit_oracle_encode(cfg_loc, flat, px, [1, 1], to)
    out_l, _ = O.vit_oracle_encode(cfg_loc, flat, px2, [1, 1], to)
    np.testing.assert_array_equal(out_l[:T], base_l[:T])      # local layers never mix tiles


def test_one_token_one_head_by_hand():
    """S = p (one patch), no CLS, H = 1: attention returns v, so a block is affine + GELU MLP."""
    cfg = tiny_cfg(image_size=4, patch_size=4, hidden=6, heads=1, mlp=5, layers_local=1, layers_global=0,
                   has_cls=0, proj_layers=1, proj_dims=(3,))
    flat = gen.make_weights(cfg, seed=7) * 10
    w = O.unpack_weights(cfg, flat)
    px = gen.make_pixels(cfg, 1, seed=8)
    out, rto = O.vit_oracle_encode(cfg, flat, px, [1], [0, 1])
    eps = cfg["ln_eps"]

    def ln(x, g_, b_):
        m = sum(x) / len(x)
        var = sum((t - m) ** 2 for t in x) / len(x)
        return np.array([(t - m) / math.sqrt(var + eps) for t in x]) * g_ + b_

    lw = w["layers"][0]
    x = w["patch_w"] @ px[0].astype(np.float64).reshape(-1) + w["patch_b"] + w["pos"][0]
    h = ln(x, lw["ln1_g"], lw["ln1_b"])
    v = lw["wqkv"][12:18] @ h + lw["bqkv"][12:18]
    x = x + lw["wo"] @ v + lw["bo"]
    h = ln(x, lw["ln2_g"], lw["ln2_b"])
    u = lw["w1"] @ h + lw["b1"]
    u = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u])
    x = x + lw["w2"] @ u + lw["b2"]
    x = ln(x, w["lnf_g"], w["lnf_b"])
    y = w["proj"][0][0] @ x + w["proj"][0][1]
    np.testing.assert_allclose(out[0], y, rtol=1e-12, atol=1e-13)
    assert list(rto) == [0, 1]


def test_packing_invariance_bitwise():
    cfg = tiny_cfg()
    flat = gen.make_weights(cfg, seed=0)
    tpi = [1, 3, 2, 1]
    to, px = _small_inputs(cfg, tpi)
    T = O.tokens_per_tile(cfg)
    ref, rto = O.vit_oracle_encode(cfg, flat, px, [1, 0, 2, 1], to)
    assert list(rto) == [0, T, T, 6 * T, 7 * T]
    # repack across requests: same images, different request split
    alt, rto2 = O.vit_oracle_encode(cfg, flat, px, [4], to)
    np.testing.assert_array_equal(alt, ref)
    assert list(rto2) == [0, 7 * T]
    # reorder images
    perm = [2, 0, 3, 1]
    tiles = [list(range(to[i], to[i + 1])) for i in range(4)]
    px_p = np.concatenate([px[tiles[i]] for i in perm])
    to_p = np.concatenate([[0], np.cumsum([tpi[i] for i in perm])])
    out_p, _ = O.vit_oracle_encode(cfg, flat, px_p, [2, 2], to_p)
    for j, i in enumerate(perm):
        np.testing.assert_array_equal(out_p[to_p[j] * T:to_p[j + 1] * T], ref[to[i] * T:to[i + 1] * T])
    # each image alone
    for i in range(4):
        one, _ = O.vit_oracle_encode(cfg, flat, px[tiles[i]], [1], [0, tpi[i]])
        np.testing.assert_array_equal(one, ref[to[i] * T:to[i + 1] * T])
    # sampled images only
    part, _ = O.vit_oracle_encode(cfg, flat, px, [4], to, images=[1])
    np.testing.assert_array_equal(part[to[1] * T:to[2] * T], ref[to[1] * T:to[2] * T])
    assert np.isnan(part[:to[1] * T]).all()


def test_fp32_vs_fp64_small():
    cfg = gen.get_config("test_medium_fp32")
    flat = gen.make_weights(cfg, seed=0)
    to, px = _small_inputs(cfg, [2, 1])
    a, _ = O.vit_oracle_encode(cfg, flat, px, [2], to, dtype=np.float64)
    b, _ = O.vit_oracle_encode(cfg, flat, px, [2], to, dtype=np.float32)
    assert b.dtype == np.float32
    rel = np.abs(a - b).max(-1) / np.abs(a).max(-1)
    assert rel.max() < 1e-4


def test_argument_validation():
    cfg = tiny_cfg()
    flat = gen.make_weights(cfg)
    px = gen.make_pixels(cfg, 2)
    with pytest.raises(ValueError):
        O.vit_oracle_encode(cfg, flat, px, [1], [0, 1, 2])        # two images announced by offsets, one by requests
    with pytest.raises(ValueError):
        O.vit_oracle_encode(cfg, flat, px, [2], [0, 2, 2])        # image without tiles
    with pytest.raises(ValueError):
        O.vit_oracle_encode(cfg, flat[:-1], px, [2], [0, 1, 2])
    out, rto = O.vit_oracle_encode(cfg, flat, px[:0], [0, 0], [0])
    assert out.shape == (0, 160) and list(rto) == [0, 0, 0]


def test_weight_layout_agrees_with_generator():
    for name in ("cfg1_tiny_fp32", "test_dh72_bf16", "test_dh80_bf16", "test_small_bf16"):
        cfg = gen.get_config(name)
        flat = gen.make_weights(cfg)
        assert flat.size == gen.weight_count(cfg)
        O.unpack_weights(cfg, flat)     # raises if the two disagree on the total
