"""The allocation-free entry point against the ordinary one: same kernels, workspace in the library's static
device array, attention work lists written by a kernel.  Two calls in a row, the second smaller, so that
whatever the first call left in the array is there when the second runs."""
import numpy as np
import pytest

import gen
from parity_util import say

pytestmark = pytest.mark.gpu


def _both(V, torch, enc, cfg, tiles_per_image, ipr, pseed):
    to = np.concatenate([[0], np.cumsum(tiles_per_image)]).astype(np.int32)
    px = torch.from_numpy(gen.make_pixels(cfg, int(to[-1]), seed=pseed)).cuda()
    want, rto_want = enc.encode(px, ipr, to)
    n_tok, out_dim, out_bytes, ws_bytes = enc.query(int(to[-1]), len(tiles_per_image))
    assert ws_bytes <= V.binding.VIT_STATIC_SCRATCH_BYTES
    got = torch.full_like(want, float("nan"))
    stream = torch.cuda.current_stream().cuda_stream
    rto = V.vit_encode_packed_static(enc.handle, px.data_ptr(), ipr, to, got.data_ptr(), out_bytes, stream)
    torch.cuda.synchronize()
    assert list(rto) == list(rto_want)
    assert torch.isfinite(got.float()).all()
    same = torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                       want.view(torch.int16 if want.dtype == torch.bfloat16 else torch.int32))
    say(f"    static vs workspace: tiles={int(to[-1])} images={len(tiles_per_image)} tokens={n_tok} bitwise equal={same}")
    assert same
    return got


@pytest.mark.parametrize("name", ["test_medium_bf16", "test_small_fp32"])
def test_static_scratch_entry_point_matches_workspace_entry_point(name):
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config(name)  # local + global layers, CLS, two-layer projector
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        _both(V, torch, enc, cfg, [2, 1, 3, 1], [2, 0, 1, 1], pseed=1)   # 7 tiles, ragged global segments
        _both(V, torch, enc, cfg, [1, 2], [2], pseed=2)                  # then a smaller batch
    finally:
        enc.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_medium_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        n = 1
        while enc.query(n, n)[3] <= V.binding.VIT_STATIC_SCRATCH_BYTES:
            n *= 2
        px = torch.zeros((n,) + (cfg["channels"], cfg["image_size"], cfg["image_size"]), device="cuda")
        n_tok, out_dim, out_bytes, _ = enc.query(n, n)
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(V.VitError) as e:
            V.vit_encode_packed_static(enc.handle, px.data_ptr(), [n], np.arange(n + 1), out.data_ptr(), out_bytes, 0)
        assert e.value.status == V.binding.VIT_ECAPACITY and "static scratch" in str(e.value)
    finally:
        enc.close()


def test_static_scratch_entry_point_refuses_too_many_images():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_small_bf16")  # 17 tokens per tile: 257 images fit the array many times over
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        m = V.binding.VIT_STATIC_MAX_IMAGES + 1
        n_tok, out_dim, out_bytes, ws_bytes = enc.query(m, m)
        assert ws_bytes <= V.binding.VIT_STATIC_SCRATCH_BYTES
        px = torch.zeros((m, cfg["channels"], cfg["image_size"], cfg["image_size"]), device="cuda")
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(V.VitError) as e:
            V.vit_encode_packed_static(enc.handle, px.data_ptr(), [m], np.arange(m + 1), out.data_ptr(), out_bytes, 0)
        assert e.value.status == V.binding.VIT_ECAPACITY and "images" in str(e.value)
        # one image fewer is taken
        out.fill_(float("nan"))
        V.vit_encode_packed_static(enc.handle, px.data_ptr(), [m - 1], np.arange(m), out.data_ptr(), out_bytes, 0)
        torch.cuda.synchronize()
        assert torch.isfinite(out[: (m - 1) * 17].float()).all()
    finally:
        enc.close()
