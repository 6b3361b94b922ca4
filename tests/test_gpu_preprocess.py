"""GPU preprocessing (resize, rescale, normalise, tile; Sec. 2 "Image Preprocessing") through the C ABI
against its CPU oracle.

Tolerance.  The kernel computes source coordinates and weights in fp32, the oracle in fp64.  A coordinate
o * in/out carries a relative rounding error of 2^-24 per operation, about 1e-7 * o pixels; the output
moves by at most that times the largest tap difference (255) times the scale 1 / (255 * std), taken
four times over for the operations involved: atol = 4e-7 * canvas side / min(std) + 2e-6 (the second term
for the fp32 evaluation of the blend itself).  The bilinear surface is continuous, so a tap index that
flips at an integer coordinate moves nothing."""
import numpy as np
import pytest

import gen
from oracle import preprocess_oracle as P
from parity_util import assert_parity, say

pytestmark = pytest.mark.gpu

MEAN, STD = (0.48, 0.45, 0.41, 0.5), (0.27, 0.26, 0.28, 0.25)


def run(img, S, rows, cols, thumb):
    import torch

    import paper_2502_00937_amd as V

    c = img.shape[2]
    out = V.preprocess_tiles(torch.from_numpy(img).cuda(), S, rows, cols, thumb, MEAN[:c], STD[:c])
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("H,W,C,S,rows,cols,thumb", [
    (37, 53, 3, 16, 2, 3, True),      # upsample, ragged source
    (200, 120, 3, 28, 2, 1, True),    # shrink one axis, stretch the other
    (64, 64, 1, 32, 2, 2, False),     # same size: the resize is the identity
    (90, 41, 4, 24, 1, 3, True),
    (896, 896, 3, 448, 2, 2, True),   # Table 1's example image: 4 tiles + 1 thumbnail = 5
    (1, 1, 3, 8, 1, 1, True),         # a single pixel stretched over everything
])
def test_preprocess_matches_oracle(H, W, C, S, rows, cols, thumb):
    say(f"case preprocess {H}x{W}x{C} -> {rows}x{cols} tiles of {S}, thumbnail={thumb}")
    img = gen.make_image_u8(H, W, C, seed=H + W)
    got = run(img, S, rows, cols, thumb)
    want = P.preprocess_tiles(img, S, rows, cols, thumb, MEAN[:C], STD[:C])
    assert got.shape == want.shape and got.dtype == np.float32
    err = np.abs(got - want).max()
    atol = 4e-7 * max(rows * S, cols * S) / min(STD[:C]) + 2e-6
    say(f"    max abs err {err:.3e} (bound {atol:.1e})")
    assert err <= atol
    if (H, W) == (rows * S, cols * S):   # identity resize: only the final multiply-add rounds
        assert np.abs(got[:rows * cols] - want[:rows * cols]).max() <= 1e-6


def test_preprocess_feeds_the_encoder():
    """Raw image -> GPU preprocessing -> encoder, against oracle preprocessing -> oracle encoder."""
    import torch

    import paper_2502_00937_amd as V
    from oracle import vit_oracle as O

    cfg = gen.get_config("test_small_bf16")     # 56-px tiles
    S = cfg["image_size"]
    img = gen.make_image_u8(150, 97, 3, seed=11)
    say("case preprocess -> encode (2 x 2 tiles + thumbnail = one image of 5 tiles)")
    px = V.preprocess_tiles(torch.from_numpy(img).cuda(), S, 2, 2, True, MEAN[:3], STD[:3])
    weights = gen.make_weights(cfg, seed=0)
    enc = V.VitEncoder(cfg, weights, device=0)
    out, _ = enc.encode(px, [1], [0, 5])
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    enc.close()
    px_want = P.preprocess_tiles(img, S, 2, 2, True, MEAN[:3], STD[:3])
    want, _ = O.vit_oracle_encode(cfg, weights, px_want, [1], [0, 5])
    assert_parity(got, want, "bf16", "preprocess+encode")


def test_preprocess_capacity_error_launches_nothing():
    import torch

    import paper_2502_00937_amd as V

    img = torch.zeros((8, 8, 3), dtype=torch.uint8, device="cuda")
    out = torch.full((1, 3, 4, 4), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(V.VitError) as e:
        V.vit_preprocess_tiles(img.data_ptr(), 8, 8, 3, 4, 1, 1, True, MEAN[:3], STD[:3], out.data_ptr(), out.numel() * 4)
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert (out == 7.0).all()
