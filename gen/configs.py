"""Encoder shape presets.

The paper names the encoder only as a vision transformer (Sec. 2, "Image
Encoding") and lists tile sizes and tokens per tile in Table 1 (560x560 tiles ->
1601 tokens, 384x384 -> 729 tokens).  The five workload shapes below follow the
benchmark definition of this repository; the small ones are test shapes.

A config is a plain dict; keys mirror the fields of ``vit_config_t`` in
``include/vitenc.h``.
"""
from __future__ import annotations

_KEYS = (
    "image_size", "patch_size", "channels", "hidden", "heads", "mlp",
    "layers_local", "layers_global", "has_cls", "final_ln", "ln_eps",
    "proj_layers", "proj_dims", "dtype", "token_merge",
)


def _cfg(image_size, patch_size, hidden, heads, mlp, layers_local, layers_global=0,
         has_cls=1, final_ln=1, ln_eps=1e-6, proj_dims=(), dtype="bf16", channels=3, token_merge=1):
    proj_dims = tuple(int(d) for d in proj_dims)
    assert len(proj_dims) <= 2
    return {
        "image_size": image_size, "patch_size": patch_size, "channels": channels,
        "hidden": hidden, "heads": heads, "mlp": mlp,
        "layers_local": layers_local, "layers_global": layers_global,
        "has_cls": has_cls, "final_ln": final_ln, "ln_eps": ln_eps,
        "proj_layers": len(proj_dims), "proj_dims": proj_dims, "dtype": dtype,
        "token_merge": token_merge,
    }


CONFIGS = {
    # 1: tiny fp32 ViT, 224 px, patch 16 -> 196 + CLS = 197 tokens
    "cfg1_tiny_fp32": _cfg(224, 16, 192, 3, 768, 12, dtype="fp32"),
    # 2/3: CLIP-style ViT-L/14 at 336 px -> 576 + CLS = 577 tokens, 2-layer GELU projector
    "cfg2_vitl14_336": _cfg(336, 14, 1024, 16, 4096, 24, proj_dims=(4096, 4096)),
    # 4: SigLIP-style, 384 px, patch 14 -> floor(384/14)^2 = 729 tokens, no CLS (Table 1)
    "cfg4_siglip_384": _cfg(384, 14, 1152, 16, 4304, 27, has_cls=0, proj_dims=(4096, 4096)),
    # 5: ViT-H/14 at 560 px tiles -> 1600 + CLS = 1601 tokens per tile (Table 1),
    #    32 tile-local layers then 8 layers attending over all tiles of an image
    "cfg5_vith14_560": _cfg(560, 14, 1280, 16, 5120, 32, layers_global=8),
    # 6 (second workload): a 6 B-class encoder on 448-px tiles whose 32 x 32 patch tokens are down-sampled
    #    2 x 2 to the 256 tokens per tile of Table 1 (5 x 256 = 1280 per image).  The paper names the size
    #    class only; width, depth and the projector widths are this repository's choice for that class
    #    (45 blocks of hidden 3200 = 25 heads of 128, MLP 12800: 5.5 G parameters; projector 12800 -> 6144 -> 6144).
    "cfg6_6b_448": _cfg(448, 14, 3200, 25, 12800, 45, proj_dims=(6144, 6144), token_merge=2),
    # ---- small test shapes (not benchmark workloads) ----
    # head dim 64, CLS, local+global, 2-layer projector, odd patch count
    "test_small_bf16": _cfg(56, 14, 128, 2, 256, 2, layers_global=1, proj_dims=(192, 160)),
    "test_small_fp32": _cfg(56, 14, 128, 2, 256, 2, layers_global=1, proj_dims=(192, 160), dtype="fp32"),
    # head dim 72 (9 x 8), no CLS, image side not a multiple of the patch (60 = 4*14 + 4), 1-layer projector
    "test_dh72_bf16": _cfg(60, 14, 144, 2, 272, 2, has_cls=0, proj_dims=(96,)),
    # head dim 80, CLS, local + global layers, no projector, no final LN
    "test_dh80_bf16": _cfg(70, 14, 160, 2, 320, 1, layers_global=2, final_ln=0),
    # head dims 96 and 128 (the remaining attention instantiations)
    "test_dh96_bf16": _cfg(56, 14, 192, 2, 384, 1, layers_global=1, proj_dims=(64,)),
    "test_dh128_bf16": _cfg(56, 14, 256, 2, 512, 2, has_cls=0),
    # several key tiles per segment and a ragged tail: 15x15 + 1 = 226 tokens per tile
    "test_medium_bf16": _cfg(210, 14, 256, 4, 512, 2, layers_global=1, proj_dims=(256, 128)),
    "test_medium_fp32": _cfg(210, 14, 256, 4, 512, 2, layers_global=1, proj_dims=(256, 128), dtype="fp32"),
    # odd numbers of 64-wide k-stages (1, 3, 5) and one, two and three tile columns: 14x14 + 1 = 197 tokens
    "test_oddk_bf16": _cfg(56, 4, 192, 3, 320, 2),
    # token down-sampling: 8 x 8 patches + CLS = 65 tokens per tile -> 4 x 4 = 16 output tokens of 4 * 128
    # channels, 2-layer projector; without CLS, no projector and 3 x 3 blocks (g = 6 -> 2 x 2 = 4 tokens of 9 * 64)
    "test_merge_bf16": _cfg(56, 7, 128, 2, 256, 1, layers_global=1, proj_dims=(192, 160), token_merge=2),
    "test_merge_fp32": _cfg(56, 7, 128, 2, 256, 1, layers_global=1, proj_dims=(192, 160), token_merge=2, dtype="fp32"),
    "test_merge3_bf16": _cfg(60, 10, 64, 1, 128, 2, has_cls=0, final_ln=0, token_merge=3),
}


def get_config(name: str) -> dict:
    cfg = dict(CONFIGS[name])
    assert tuple(cfg.keys()) == _KEYS
    return cfg


def tokens_per_tile(cfg: dict) -> int:
    """Tokens one tile yields: floor(S/p)^2 patches plus one CLS row if present (Table 1)."""
    g = cfg["image_size"] // cfg["patch_size"]
    return g * g + (1 if cfg["has_cls"] else 0)


def out_tokens_per_tile(cfg: dict) -> int:
    """Tokens one tile hands on: all of them, or (g / m)^2 after m x m token down-sampling
    (Table 1: 448-px tiles -> 256 tokens)."""
    m = cfg["token_merge"]
    if m <= 1:
        return tokens_per_tile(cfg)
    g = cfg["image_size"] // cfg["patch_size"]
    assert g % m == 0
    return (g // m) ** 2


def weight_layout(cfg: dict):
    """Ordered (name, shape) list of the flat fp32 weight buffer (the interchange format).

    Matrices are stored [out_features, in_features]; the patch matrix is the
    convolution kernel [hidden, channels, p, p] flattened over (c, py, px).
    """
    D, M = cfg["hidden"], cfg["mlp"]
    K = cfg["channels"] * cfg["patch_size"] ** 2
    T = tokens_per_tile(cfg)
    out = [("patch_w", (D, K)), ("patch_b", (D,))]
    if cfg["has_cls"]:
        out.append(("cls", (D,)))
    out.append(("pos", (T, D)))
    for l in range(cfg["layers_local"] + cfg["layers_global"]):
        p = f"l{l}."
        out += [
            (p + "ln1_g", (D,)), (p + "ln1_b", (D,)),
            (p + "wqkv", (3 * D, D)), (p + "bqkv", (3 * D,)),
            (p + "wo", (D, D)), (p + "bo", (D,)),
            (p + "ln2_g", (D,)), (p + "ln2_b", (D,)),
            (p + "w1", (M, D)), (p + "b1", (M,)),
            (p + "w2", (D, M)), (p + "b2", (D,)),
        ]
    if cfg["final_ln"]:
        out += [("lnf_g", (D,)), ("lnf_b", (D,))]
    d_in = D * max(cfg["token_merge"], 1) ** 2
    for i in range(cfg["proj_layers"]):
        d_out = cfg["proj_dims"][i]
        out += [(f"proj{i}_w", (d_out, d_in)), (f"proj{i}_b", (d_out,))]
        d_in = d_out
    return out


def weight_count(cfg: dict) -> int:
    n = 0
    for _, shape in weight_layout(cfg):
        k = 1
        for s in shape:
            k *= s
        n += k
    return n
