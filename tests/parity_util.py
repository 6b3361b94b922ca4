"""Helpers shared by the GPU parity tests: run the HIP library and the oracle on the same seeded inputs."""
import time

import numpy as np

import gen
from oracle import vit_oracle as O

# Parity bar of this project for bf16 arithmetic: per token, max-norm error relative to the
# token's max-norm, and cosine similarity.  fp32 arithmetic is held to a tighter bar that
# reflects fp32 accumulation over at most ~5000-term dot products and a dozen layers.
BF16_REL, BF16_COS = 2e-2, 0.999
FP32_REL, FP32_COS = 2e-4, 0.999999


def say(msg):
    import conftest

    conftest.progress(msg)


def token_metrics(got: np.ndarray, want: np.ndarray):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), "non-finite values in the GPU output"
    rel = np.abs(got - want).max(-1) / np.abs(want).max(-1)
    cos = (got * want).sum(-1) / (np.linalg.norm(got, axis=-1) * np.linalg.norm(want, axis=-1))
    return float(rel.max()), float(cos.min())


def assert_parity(got, want, dtype: str, label=""):
    rel, cos = token_metrics(got, want)
    say(f"    parity {label}: tokens={got.shape[0]} max rel={rel:.3e} min cos={cos:.7f}")
    if dtype == "bf16":
        assert rel <= BF16_REL and cos >= BF16_COS, (label, rel, cos)
    else:
        assert rel <= FP32_REL and cos >= FP32_COS, (label, rel, cos)
    return rel, cos


def gpu_encode(cfg, weights, px, ipr, tile_offsets, enc=None):
    import torch

    import paper_2502_00937_amd as V

    own = enc is None
    if own:
        enc = V.VitEncoder(cfg, weights, device=0)
    out, rto = enc.encode(torch.from_numpy(px).cuda(), ipr, tile_offsets)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    if own:
        enc.close()
    return got, rto


def check_case(cfg, tiles_per_image, ipr, wseed=0, pseed=1, wscale=1.0, oracle_dtype=np.float64, images=None,
               label=""):
    """Encode on the GPU (whole batch) and with the oracle (whole batch or sampled images); compare."""
    weights = gen.make_weights(cfg, seed=wseed)
    if wscale != 1.0:
        weights = weights * np.float32(wscale)
        if cfg["dtype"] == "bf16":
            weights = gen.round_to_bf16(weights)
    to = np.concatenate([[0], np.cumsum(tiles_per_image)]).astype(np.int32)
    px = gen.make_pixels(cfg, int(to[-1]), seed=pseed)
    big = weights.size > (1 << 30)  # progress lines for the one case whose steps take minutes
    if big:
        say(f"    {label}: {weights.size / 1e9:.2f} G weights generated")
    t0 = time.time()
    got, rto = gpu_encode(cfg, weights, px, ipr, to)
    t1 = time.time()
    if big:
        say(f"    {label}: gpu done in {t1 - t0:.1f}s, oracle running")
    want, rto_want = O.vit_oracle_encode(cfg, weights, px, ipr, to, dtype=oracle_dtype, images=images)
    say(f"    {label}: gpu {t1 - t0:.1f}s oracle {time.time() - t1:.1f}s")
    assert list(rto) == list(rto_want)
    T = O.out_tokens_per_tile(cfg)
    if images is None:
        assert_parity(got, want, cfg["dtype"], label)
    else:
        for i in images:
            a, b = int(to[i]) * T, int(to[i + 1]) * T
            assert_parity(got[a:b], want[a:b], cfg["dtype"], f"{label} image {i}")
    return got, want
