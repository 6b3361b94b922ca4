"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The GPU encodes the whole batch; the oracle encodes whole images sampled from it (an image's
tokens depend on its own tiles only), because the full batches are 100+ TFLOP.
"""
import os

import numpy as np
import pytest

import gen
from parity_util import check_case, say

pytestmark = pytest.mark.gpu


def _workload(name):
    cfg, ipr, to = gen.make_workload(name)
    return cfg, list(ipr), list(np.diff(to))


def test_cfg1_tiny_fp32_full():
    cfg, ipr, tpi = _workload("cfg1")
    say("case cfg1 (4 images, fp32)")
    got, _ = check_case(cfg, tpi, ipr, label="cfg1")
    assert got.shape == (4 * 197, 192)


def test_cfg2_vitl14_336_full():
    cfg, ipr, tpi = _workload("cfg2")
    say("case cfg2 (8 images)")
    got, _ = check_case(cfg, tpi, ipr, label="cfg2")
    assert got.shape == (8 * 577, 4096)


def test_cfg3_ragged_batch_sampled():
    cfg, ipr, tpi = _workload("cfg3")
    # first, last, three inside the 32-image request (request 47: its first, one inside, its last), one of
    # the 26-image request, two single-image requests
    first_of_req = np.concatenate([[0], np.cumsum(ipr)])
    assert ipr[47] == 32 and ipr[48] == 26 and ipr[60] == 1 and ipr[9] == 1
    r47 = int(first_of_req[47])
    images = [0, int(first_of_req[9]), r47, r47 + 17, r47 + 31, int(first_of_req[48]) + 12, int(first_of_req[60]), 259]
    say(f"case cfg3 (260 images / 64 requests), oracle on images {images}")
    got, _ = check_case(cfg, tpi, ipr, images=images, label="cfg3")
    assert got.shape == (260 * 577, 4096)


def test_cfg4_siglip_tiles_sampled():
    cfg, ipr, tpi = _workload("cfg4")
    images = [0, 5, 64, 127]   # the first image (7 tiles, the maximum), a 2-tile one, one inside, the last (5 tiles)
    assert tpi[0] == 7 and tpi[5] == 2 and tpi[127] == 5
    say(f"case cfg4 (128 images / 591 tiles), oracle on images {images}")
    got, _ = check_case(cfg, tpi, ipr, images=images, oracle_dtype=np.float32, label="cfg4")
    assert got.shape == (591 * 729, 4096)


def test_cfg5_local_global_sampled():
    cfg, ipr, tpi = _workload("cfg5")
    images = [31]
    say(f"case cfg5 (32 images x 4 tiles), oracle on image {images}")
    got, _ = check_case(cfg, tpi, ipr, images=images, oracle_dtype=np.float32, label="cfg5")
    assert got.shape == (128 * 1601, 1280)


@pytest.mark.skipif(os.environ.get("VITENC_SKIP_6B") == "1",
                    reason="VITENC_SKIP_6B=1: the second workload at full size needs 5.65 G weights (23 GB fp32, "
                           "34 GB of host memory at the peak, a minute to generate) and a 12 TFLOP fp32 oracle pass")
def test_cfg6_6b_downsampled_sampled():
    cfg, ipr, tpi = _workload("cfg6")
    images = [7]               # the single-tile image
    assert tpi[7] == 1
    say(f"case cfg6 (8 images / 36 tiles, 6B-class, 2x2 down-sampling), oracle on image {images}")
    got, _ = check_case(cfg, tpi, ipr, images=images, oracle_dtype=np.float32, label="cfg6")
    assert got.shape == (36 * 256, 6144)


def test_tokens_are_bit_identical_at_every_batch_size():
    """An image's tokens do not depend on how many images share its launch: 1, 2, 3 and 8 images run every
    product on the ring kernel (four- and two-stage rings; 1 to 3 images with its 64-row tiles for the
    narrow products, 8 images with three two-stage workgroups of 64 rows to a unit for them),
    64 images mix both matrix-product kernels, 260 images run the persistent 256 x 256
    kernel, and all of them add a token's k-steps in the same order.  Compared bit for bit against the
    full config-3 batch."""
    import torch

    import paper_2502_00937_amd as V

    cfg, ipr, tpi = _workload("cfg3")
    say("case batch-size invariance (config-3 model: 260, 64, 8, 3, 2, 1 images)")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    px = torch.from_numpy(gen.make_pixels(cfg, 260, seed=1)).cuda()
    T = gen.tokens_per_tile(cfg)
    full, _ = enc.encode(px, ipr, np.arange(261, dtype=np.int32))
    torch.cuda.synchronize()
    for n in (64, 8, 3, 2, 1):
        part, _ = enc.encode(px[:n], [n], np.arange(n + 1, dtype=np.int32))
        torch.cuda.synchronize()
        same = torch.equal(part.view(torch.int16), full[:n * T].view(torch.int16))
        say(f"    {n} images against the first {n} of 260: bit-identical = {same}")
        assert same, n
    # images from the far end of the batch, encoded alone
    tail, _ = enc.encode(px[257:], [3], np.arange(4, dtype=np.int32))
    torch.cuda.synchronize()
    assert torch.equal(tail.view(torch.int16), full[257 * T:].view(torch.int16))
    enc.close()


def test_buffers_of_more_than_2_31_elements():
    """The config-4 encoder over 700 tiles (510 300 tokens): the fc1 output holds 2.22e9 elements and the QKV
    buffer 1.96e9, so element indices pass 2^31 and byte offsets 2^32 in every large buffer.  The first image and
    the last one (the highest rows of every buffer) are compared with the oracle."""
    cfg = gen.get_config("cfg4_siglip_384")
    tpi = [5] * 140
    T = gen.tokens_per_tile(cfg)
    assert sum(tpi) * T * 4352 > 2 ** 31 and sum(tpi) * T < 2 ** 31 - 1024
    say(f"case 2^31 elements: {sum(tpi)} tiles, {sum(tpi) * T} tokens")
    got, _ = check_case(cfg, tpi, [1] * len(tpi), images=[0, 139], oracle_dtype=np.float32, label="2^31")
    assert got.shape == (sum(tpi) * T, 4096)


def test_head_by_head_qkv_buffer_past_4_gib():
    """Head dim 64 stores the QKV product head by head: 48 blocks of [rows, 64].  With 700 400 token rows (41 200
    tiles of 17 tokens, hidden 1024 = 16 heads) the buffer is 4.3 GB, so the last heads' blocks start past byte 2^32.
    One layer, a narrow MLP, no projector: the first and the last image against the oracle, and the last three
    images encoded alone (every product on the small-tile kernel, a 2 KB QKV buffer) bit for bit."""
    import torch

    import paper_2502_00937_amd as V

    from oracle import vit_oracle as O
    from parity_util import assert_parity

    cfg = {"image_size": 56, "patch_size": 14, "channels": 3, "hidden": 1024, "heads": 16, "mlp": 256,
           "layers_local": 1, "layers_global": 0, "has_cls": 1, "final_ln": 1, "ln_eps": 1e-6, "proj_layers": 0,
           "proj_dims": (), "dtype": "bf16", "token_merge": 1}
    n, T = 41200, 17
    assert gen.tokens_per_tile(cfg) == T and 48 * n * T * 64 * 2 > 2 ** 32
    say(f"case head-by-head QKV past 4 GiB: {n} tiles, {n * T} tokens")
    weights = gen.make_weights(cfg, seed=3)
    px = gen.make_pixels(cfg, n, seed=4)
    enc = V.VitEncoder(cfg, weights, device=0)
    try:
        dpx = torch.from_numpy(px).cuda()
        full, _ = enc.encode(dpx, [n], np.arange(n + 1, dtype=np.int32))
        torch.cuda.synchronize()
        assert full.shape == (n * T, 1024)
        tail, _ = enc.encode(dpx[n - 3:], [3], np.arange(4, dtype=np.int32))
        torch.cuda.synchronize()
        same = torch.equal(tail.view(torch.int16), full[(n - 3) * T:].view(torch.int16))
        say(f"    last three images alone against the batch: bit-identical = {same}")
        assert same
        for i in (0, n - 1):
            want, _ = O.vit_oracle_encode(cfg, weights, px[i:i + 1], [1], np.array([0, 1], dtype=np.int32))
            assert_parity(full[i * T:(i + 1) * T].float().cpu().numpy(), want, "bf16", f"4 GiB image {i}")
    finally:
        enc.close()
