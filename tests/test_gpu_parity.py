"""GPU parity: the HIP library through its C ABI against the CPU oracle, on seeded inputs."""
import numpy as np
import pytest

import gen
from oracle import vit_oracle as O
from parity_util import assert_parity, check_case, gpu_encode, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,tpi,ipr", [
    ("test_small_fp32", [1, 3, 2], [1, 0, 2]),
    ("test_small_bf16", [1, 3, 2], [1, 0, 2]),
    ("test_dh72_bf16", [2, 1, 1], [3]),
    ("test_dh80_bf16", [3, 1], [1, 1]),
    ("test_medium_fp32", [2, 1], [2]),
    ("test_medium_bf16", [2, 1, 4], [1, 1, 1]),
    ("test_dh96_bf16", [2, 1, 3], [2, 1]),
    ("test_dh128_bf16", [1, 2, 1], [1, 2]),
])
def test_small_configs_match_oracle(name, tpi, ipr):
    say(f"case {name} tiles_per_image={tpi} images_per_request={ipr}")
    check_case(gen.get_config(name), tpi, ipr, label=name)


@pytest.mark.parametrize("name,scale", [("test_medium_bf16", 2.0), ("test_dh80_bf16", 2.0), ("test_medium_fp32", 3.0)])
def test_large_weights_sharpen_attention(name, scale):
    """Scaled-up weights push softmax away from uniform and GELU away from linear.

    bf16 cases use x2: at x4 this network amplifies bf16 operand rounding itself beyond the bar
    (tests/test_bf16_rounding_emulation.py shows it on the CPU with no kernel involved: 0.3 ... 0.8 relative
    error from the roundings alone), so x4 would test the conditioning of the synthetic network, not
    the kernels.  fp32 arithmetic has more headroom and runs x3; at x4 it leaves its own, tighter bar as well:
    the oracle evaluated in fp32 differs from itself in fp64 by 2.5e-4 there (same CPU test)."""
    say(f"case {name} weights x{scale}")
    check_case(gen.get_config(name), [2, 3], [2], wscale=scale, label=f"{name} x{scale}")


@pytest.mark.parametrize("name,tpi,ipr", [
    ("test_merge_bf16", [1, 3, 2], [2, 0, 1]),     # 2 x 2 down-sampling, CLS dropped, 2-layer projector
    ("test_merge_fp32", [2, 1], [1, 1]),
    ("test_merge3_bf16", [1, 2, 1, 4], [4]),        # 3 x 3, no CLS, no final LN, no projector: straight to the output
])
def test_token_downsampling_matches_oracle(name, tpi, ipr):
    """Token down-sampling between the final LayerNorm and the projector (Table 1: 448-px tiles -> 256 tokens)."""
    cfg = gen.get_config(name)
    say(f"case {name} tiles/image {tpi}")
    got, want = check_case(cfg, tpi, ipr, label=name)
    assert got.shape == (sum(tpi) * gen.out_tokens_per_tile(cfg), want.shape[1])


def test_token_downsampling_many_tiles_bf16():
    """A 448-px-style grid at reduced width: 16 x 16 patches + CLS = 257 tokens per tile -> 64 output tokens
    of 4 * 256 channels; 40 tiles, so the projector's operand has several row tiles and a ragged tail."""
    cfg = gen.get_config("test_merge_bf16")
    cfg.update(image_size=112, hidden=256, heads=4, mlp=512, proj_dims=(320, 192))
    tpi = [5, 1, 5, 3, 5, 1, 5, 5, 5, 5]
    say("case down-sampling, 40 tiles")
    got, _ = check_case(cfg, tpi, [3, 0, 7], images=[0, 1, 3, 9], label="merge40")
    assert got.shape == (40 * 64, 192)


def test_maximum_width():
    """The widest encoder the library accepts: hidden 4096 (the LayerNorm's register budget), 32 heads of
    128, MLP 8192 (128 k-stages), a 2 x 2 patch grid; one block keeps the weights at 0.2 G."""
    cfg = gen.get_config("test_dh128_bf16")
    cfg.update(image_size=28, patch_size=14, hidden=4096, heads=32, mlp=8192, layers_local=1, layers_global=0,
               has_cls=1, proj_layers=1, proj_dims=(4096,))
    say("case maximum width (hidden 4096, 32 heads of 128, MLP 8192)")
    check_case(cfg, [2, 1, 3], [1, 2], label="max width")
    import paper_2502_00937_amd as V

    assert V.vit_weight_count(dict(cfg, hidden=4104, heads=27)) == 0   # 27 heads of 152: beyond both limits


def test_ragged_many_tiles_bf16():
    """Enough rows for several 256-row GEMM tiles plus a ragged tail; heavy-tailed request sizes."""
    cfg = gen.get_config("test_medium_bf16")          # 226 tokens per tile
    tpi = [1, 5, 1, 1, 2, 7, 1, 3]                     # 21 tiles -> 4746 rows
    say("case ragged 21 tiles")
    check_case(cfg, tpi, [1, 0, 4, 3], label="ragged")


def test_wide_batch_mixes_both_gemm_kernels():
    """160 tiles x 226 = 36 160 token rows (142 row blocks of 256, ragged last one): the QKV product (three tile
    columns, 426 tiles) takes the persistent 256 x 256 kernel, the others (one or two tile columns) the
    128 x 128 ring kernel with two-stage rings; K of 4 and 8 k-stages.  The oracle encodes sampled images
    (first, a multi-tile one, last)."""
    cfg = gen.get_config("test_medium_bf16")
    tpi = [1, 4, 1, 1, 2, 7, 1, 3] * 8           # 64 images, 160 tiles
    say("case wide batch (160 tiles, both GEMM kernels)")
    got, _ = check_case(cfg, tpi, [len(tpi)], images=[0, 5, 63], label="wide")
    assert got.shape[0] == 160 * 226


def test_odd_k_stage_counts_and_narrow_column_bands_on_the_persistent_gemm():
    """500 tiles x 197 tokens = 98 500 rows (385 row blocks), so even the products with a single tile column
    reach the persistent kernel's threshold of 384 tiles.  K = 64, 192 and 320 are 1, 3 and 5 k-stages: the two
    LDS stages change roles from one tile to the next.  N = 576, 192 and 320 are three, one and two tile
    columns: a band with an idle column and the 32 x 1 and 16 x 2 tile groups."""
    cfg = gen.get_config("test_oddk_bf16")
    tpi = [1] * 500
    say("case odd k-stage counts (500 tiles, persistent GEMM)")
    got, _ = check_case(cfg, tpi, [len(tpi)], images=[0, 171, 499], label="oddk")
    assert got.shape[0] == 500 * 197


def test_short_last_rounds_of_one_and_two_column_products():
    """The same network at 390 tiles (76 830 rows, 301 row blocks).  The products one tile column wide are walked in
    rounds of 256 row blocks and those two columns wide in rounds of 128; both leave 45 row blocks for a last round
    that would idle most of the device, so those rows go to the ring kernel in a launch of their own (at either end
    of the matrix: the walk alternates its direction from one product to the next).  The oracle encodes the first
    image, one inside and the last; the first and last two images encoded alone (ring kernel only) must give the
    bits they have in the batch."""
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_oddk_bf16")
    tpi = [1] * 390
    say("case short last rounds (390 tiles, persistent + ring launches per product)")
    got, _ = check_case(cfg, tpi, [len(tpi)], images=[0, 200, 389], label="short-round")
    assert got.shape[0] == 390 * 197
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        px = torch.from_numpy(gen.make_pixels(cfg, 390, seed=1)).cuda()
        full, _ = enc.encode(px, [390], np.arange(391, dtype=np.int32))
        for lo in (0, 388):
            part, _ = enc.encode(px[lo:lo + 2], [2], np.arange(3, dtype=np.int32))
            torch.cuda.synchronize()
            same = torch.equal(part.view(torch.int16), full[lo * 197:(lo + 2) * 197].view(torch.int16))
            say(f"    images {lo}, {lo + 1} alone against the batch: bit-identical = {same}")
            assert same
    finally:
        enc.close()


def test_odd_k_stage_counts_on_the_ring_gemm():
    """The same network at 60 tiles (11 820 rows, 47 row blocks): every product takes the ring kernel, with
    1, 3 and 5 k-stages (fewer than the ring is deep) and rings of four and of two stages."""
    cfg = gen.get_config("test_oddk_bf16")
    tpi = [1] * 60
    say("case odd k-stage counts (60 tiles, ring GEMM)")
    got, _ = check_case(cfg, tpi, [len(tpi)], images=[0, 31, 59], label="oddk-ring")
    assert got.shape[0] == 60 * 197


def test_packing_invariance_on_gpu():
    """Reordering images / re-splitting requests must not change an image's tokens (beyond parity)."""
    cfg = gen.get_config("test_medium_bf16")
    weights = gen.make_weights(cfg, seed=0)
    tpi = [2, 1, 3]
    to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
    px = gen.make_pixels(cfg, 6, seed=1)
    T = gen.tokens_per_tile(cfg)
    say("case packing invariance")
    a, rto_a = gpu_encode(cfg, weights, px, [3], to)
    b, rto_b = gpu_encode(cfg, weights, px, [1, 1, 1], to)
    assert np.array_equal(a, b)
    assert list(rto_a) == [0, 6 * T] and list(rto_b) == [0, 2 * T, 3 * T, 6 * T]
    perm = [2, 0, 1]
    tiles = [list(range(to[i], to[i + 1])) for i in range(3)]
    px_p = np.concatenate([px[tiles[i]] for i in perm])
    to_p = np.concatenate([[0], np.cumsum([tpi[i] for i in perm])]).astype(np.int32)
    c, _ = gpu_encode(cfg, weights, px_p, [2, 1], to_p)
    bitwise = True
    for j, i in enumerate(perm):
        ca, aa = c[to_p[j] * T:to_p[j + 1] * T], a[to[i] * T:to[i + 1] * T]
        bitwise &= bool(np.array_equal(ca, aa))
        assert_parity(ca, aa, "bf16", f"permuted image {i}")
    say(f"    bitwise invariant under image permutation: {bitwise}")


def test_empty_and_text_only_requests():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_small_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg))
    px = torch.zeros((0, 3, cfg["image_size"], cfg["image_size"]), device="cuda")
    out, rto = enc.encode(px, [0, 0], [0])
    assert out.shape[0] == 0 and list(rto) == [0, 0, 0]
    out, rto = enc.encode(px, [], [0])
    assert out.shape[0] == 0 and list(rto) == [0]
    enc.close()


def test_error_paths_launch_nothing():
    import torch

    import paper_2502_00937_amd as V
    from paper_2502_00937_amd import binding as B

    cfg = gen.get_config("test_small_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg))
    S = cfg["image_size"]
    px = torch.zeros((2, 3, S, S), device="cuda")
    n_tok, out_dim, out_bytes, ws_bytes = enc.query(2, 2)
    out = torch.full((n_tok, out_dim), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(V.VitError) as ei:      # output too small
        V.vit_encode_packed(enc.handle, px.data_ptr(), [2], [0, 1, 2], out.data_ptr(), out_bytes - 2, ws.data_ptr(),
                            ws_bytes)
    assert ei.value.status == B.VIT_ECAPACITY
    with pytest.raises(V.VitError) as ei:      # workspace too small
        V.vit_encode_packed(enc.handle, px.data_ptr(), [2], [0, 1, 2], out.data_ptr(), out_bytes, ws.data_ptr(),
                            ws_bytes - 256)
    assert ei.value.status == B.VIT_ECAPACITY
    with pytest.raises(V.VitError) as ei:      # image without tiles
        V.vit_encode_packed(enc.handle, px.data_ptr(), [2], [0, 2, 2], out.data_ptr(), out_bytes, ws.data_ptr(),
                            ws_bytes)
    assert ei.value.status == B.VIT_EINVAL
    with pytest.raises(V.VitError) as ei:      # negative image count
        V.vit_encode_packed(enc.handle, px.data_ptr(), [-1], [0], out.data_ptr(), out_bytes, ws.data_ptr(), ws_bytes)
    assert ei.value.status == B.VIT_EINVAL
    # more token rows than the 32-bit row indices of the kernels hold: refused before anything is sized or touched
    T = gen.tokens_per_tile(cfg)
    too_many = (2 ** 31) // T + 1
    with pytest.raises(V.VitError) as ei:
        V.vit_encode_packed(enc.handle, px.data_ptr(), [1], [0, too_many], out.data_ptr(), out_bytes, ws.data_ptr(),
                            ws_bytes)
    assert ei.value.status == B.VIT_EINVAL
    with pytest.raises(V.VitError) as ei:
        enc.query(too_many, 1)
    assert ei.value.status == B.VIT_EINVAL
    assert enc.query((2 ** 31 - 2048) // T, 1)[0] == ((2 ** 31 - 2048) // T) * T   # just below the limit: sized, not run
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    enc.close()


def test_repeated_launches_are_deterministic():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_medium_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg))
    px = torch.from_numpy(gen.make_pixels(cfg, 5)).cuda()
    outs = []
    for _ in range(6):                     # more launches than staging slots
        out, _ = enc.encode(px, [2, 1], [0, 2, 3, 5])
        outs.append(out.clone())
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    enc.close()


def test_one_handle_serves_batches_of_changing_size_without_waiting():
    """Launches of very different sizes queued back to back on one handle and one stream (the workspace is
    reused, the pinned table slots cycle, both GEMM kernels and both ring depths take turns): every result
    equals, bit for bit, what a fresh handle produces for that batch alone."""
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_medium_bf16")      # 226 tokens per tile
    weights = gen.make_weights(cfg)
    px = torch.from_numpy(gen.make_pixels(cfg, 200)).cuda()
    batches = [[1], [3, 2, 1], [1] * 150, [2], [4] * 50, [1, 1], [7, 1], [1] * 200, [5]]
    say(f"case changing batch sizes {[sum(b) for b in batches]} tiles")
    enc = V.VitEncoder(cfg, weights)
    got = []
    for tpi in batches:                           # no synchronisation between the launches
        to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
        out, _ = enc.encode(px[:int(to[-1])], [len(tpi)], to)
        got.append(out)                           # a fresh output tensor per launch
    torch.cuda.synchronize()
    enc.close()
    for tpi, g in zip(batches, got):
        fresh = V.VitEncoder(cfg, weights)
        to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
        want, _ = fresh.encode(px[:int(to[-1])], [len(tpi)], to)
        torch.cuda.synchronize()
        fresh.close()
        if not torch.equal(g, want):  # say where: a stale buffer, a lost tile and a stray write look different
            d = (g.float() - want.float()).abs().max(1).values
            rows = torch.nonzero(d > 0).flatten().tolist()
            raise AssertionError(f"batch {tpi[:4]}... ({sum(tpi)} tiles): {len(rows)} of {g.shape[0]} token rows differ, "
                                 f"first {rows[:8]}, last {rows[-3:]}, largest difference {float(d.max()):.3e}")


def test_profile_counters():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_small_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg))
    px = torch.from_numpy(gen.make_pixels(cfg, 2)).cuda()
    enc.profile_enable(True)
    enc.encode(px, [2], [0, 1, 2])
    prof = enc.profile_read()
    L = cfg["layers_local"] + cfg["layers_global"]
    assert prof["gemm"][1] == 1 + 4 * L + 2 and prof["attention"][1] == L and prof["layernorm"][1] == 2 * L + 1
    assert all(v[0] > 0 for v in prof.values())
    enc.profile_enable(False)
    enc.close()


def test_mfma_ceiling_probe_reports_a_plausible_rate():
    import paper_2502_00937_amd as V

    say("case mfma ceiling probe, 0.05 s")
    t = V.vit_mfma_ceiling(0, 0.05, random_operands=True)
    c = V.vit_mfma_ceiling(0, 0.05, random_operands=False)
    say(f"    register-only MFMA loop: {t:.0f} TFLOP/s with random operands, {c:.0f} with a constant")
    assert 500.0 < t < 2600.0 and 500.0 < c < 2600.0  # below the nominal 2.5 PFLOP/s (+ clock tolerance), far above VALU rates


def test_routed_and_packed_launches_match_the_oracle_per_request():
    """Requests of 3, 1, 4 and 2 images are routed image by image over two instances (here: two launch
    queues on the one GPU), packed into launches of at most 3 images and encoded; every image's tokens
    must match the oracle's encoding of that image alone, wherever the router and the packer put it."""
    import torch

    import paper_2502_00937_amd as V
    from oracle import vit_oracle as O
    from paper_2502_00937_amd.router import ImageTokenRouter, LaunchPacker

    say("case router + packer end to end")
    cfg = gen.get_config("test_medium_bf16")
    T = gen.tokens_per_tile(cfg)
    weights = gen.make_weights(cfg, seed=0)
    requests = [[1, 2, 1], [1], [2, 1, 1, 1], [1, 3]]  # tiles per image
    n_tiles = sum(sum(r) for r in requests)
    px = gen.make_pixels(cfg, n_tiles, seed=1)
    first_tile, t0 = {}, 0
    for rid, tiles in enumerate(requests):
        for k, n in enumerate(tiles):
            first_tile[(rid, k)] = t0
            t0 += n
    router, packers = ImageTokenRouter(2, T), [LaunchPacker(), LaunchPacker()]
    for rid, tiles in enumerate(requests):
        for k, inst in enumerate(router.route(tiles)):
            packers[inst].push(rid, k, tiles[k])
    assert len(packers[0]) and len(packers[1])  # the load really is split
    enc = V.VitEncoder(cfg, weights, device=0)
    wparsed = O.unpack_weights(cfg, weights, np.float64)
    seen = 0
    for inst, p in enumerate(packers):
        while len(p):
            items, ipr, to = p.next_launch(max_images=3)
            sel = np.concatenate([np.arange(first_tile[(i.request_id, i.image_index)],
                                            first_tile[(i.request_id, i.image_index)] + i.tiles) for i in items])
            out, rto = enc.encode(torch.from_numpy(px[sel]).cuda(), ipr, to)
            torch.cuda.synchronize()
            got = out.float().cpu().numpy()
            assert rto[-1] == got.shape[0] == int(to[-1]) * T and len(rto) == len(ipr) + 1
            for j, it in enumerate(items):
                a = first_tile[(it.request_id, it.image_index)]
                want, _ = O.vit_oracle_encode(cfg, wparsed, px[a:a + it.tiles], [1], np.asarray([0, it.tiles]))
                assert_parity(got[int(to[j]) * T:int(to[j + 1]) * T], want, cfg["dtype"],
                              f"instance {inst} request {it.request_id} image {it.image_index}")
                router.complete(inst, it.tiles)
                seen += 1
    enc.close()
    assert seen == sum(len(r) for r in requests) and router.pending == [0, 0]


def test_pull_style_handoff_assembles_a_request_encoded_in_two_launches():
    """A request of four images is encoded in two launches (images 0, 2 and images 1, 3, as a router
    might split it) interleaved with another request; the consumer pulls when all four are published
    and must get exactly what one launch of the whole request produces, in image order."""
    import torch

    import paper_2502_00937_amd as V

    say("case pull-style hand-off")
    cfg = gen.get_config("test_medium_bf16")
    T = gen.tokens_per_tile(cfg)
    weights = gen.make_weights(cfg, seed=0)
    tiles = [1, 2, 1, 3]                                  # tiles per image of request 5
    to_all = np.concatenate([[0], np.cumsum(tiles)]).astype(np.int32)
    px = torch.from_numpy(gen.make_pixels(cfg, int(to_all[-1]) + 2, seed=1)).cuda()  # + a 2-tile image of request 6
    enc = V.VitEncoder(cfg, weights, device=0)
    whole, _ = enc.encode(px[:int(to_all[-1])], [4], to_all)
    torch.cuda.synchronize()

    h = V.TokenHandoff(0)
    h.expect(5, 4)
    h.expect(6, 1)
    side = torch.cuda.Stream()
    outs = []
    other = torch.arange(int(to_all[-1]), int(to_all[-1]) + 2)
    for launch, imgs in enumerate([[0, 2], [1, 3]]):
        sel = torch.cat([torch.arange(int(to_all[i]), int(to_all[i + 1])) for i in imgs] + ([other] if launch == 0 else []))
        n = [tiles[i] for i in imgs] + ([2] if launch == 0 else [])
        ipr = [1] * len(n)
        to = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        with torch.cuda.stream(side):
            out, _ = enc.encode(px[sel.cuda()].contiguous(), ipr, to)
            outs.append(out)                               # producer memory stays alive until release
            for j, i in enumerate(imgs):
                rows = out[int(to[j]) * T:int(to[j + 1]) * T]
                h.publish(5, i, rows.data_ptr(), rows.numel() * rows.element_size(), side.cuda_stream)
            if launch == 0:
                rows = out[int(to[2]) * T:int(to[3]) * T]
                h.publish(6, 0, rows.data_ptr(), rows.numel() * rows.element_size(), side.cuda_stream)
                assert h.complete(5)[0] is False and h.complete(6)[0] is True
                with pytest.raises(V.VitError):
                    h.pull(5, whole.data_ptr(), 1 << 30, 0)  # not ready: nothing is queued
    done, nbytes = h.complete(5)
    assert done and nbytes == whole.numel() * whole.element_size()
    dst = torch.empty_like(whole)
    with pytest.raises(V.VitError):
        h.pull(5, dst.data_ptr(), nbytes - 1, torch.cuda.current_stream().cuda_stream)  # too small
    got = h.pull(5, dst.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)  # waits on `side` through the events
    torch.cuda.synchronize()
    assert got == nbytes
    assert torch.equal(dst.view(torch.int16), whole.view(torch.int16))  # bitwise: packing never changes an image's tokens
    h.release(5)
    h.release(6)
    h.close()
    enc.close()


def _random_case(seed):
    """A seeded random small encoder + batch: shapes the fixed presets do not hit (odd patch grids, mlp and
    projector widths that are multiples of 8 only, every head-dim instantiation, down-sampling factors)."""
    rng = np.random.default_rng(1000 + seed)
    p = int(rng.choice([4, 7, 14]))
    g = int(rng.integers(3, 10))
    dh = int(rng.choice([64, 72, 80, 96, 128]))
    heads = int(rng.integers(1, 4))
    merge = int(rng.choice([m for m in (1, 1, 2, 3) if g % m == 0]))
    if seed % 3 == 0:  # every third case down-samples for sure
        g, merge = [(4, 2), (6, 3), (8, 2), (6, 2)][(seed // 3) % 4]
    n_proj = int(rng.integers(0, 3))
    cfg = {
        "image_size": g * p + int(rng.integers(0, p)), "patch_size": p, "channels": 3,
        "hidden": dh * heads, "heads": heads, "mlp": 8 * int(rng.integers(8, 80)),
        "layers_local": int(rng.integers(1, 3)), "layers_global": int(rng.integers(0, 2)),
        "has_cls": int(rng.integers(0, 2)), "final_ln": int(rng.integers(0, 2)), "ln_eps": 1e-6,
        "proj_layers": n_proj, "proj_dims": tuple(8 * int(rng.integers(4, 40)) for _ in range(n_proj)),
        "dtype": "fp32" if seed % 5 == 4 else "bf16", "token_merge": merge,
    }
    n_images = int(rng.integers(1, 6))
    tpi = [int(rng.integers(1, 5)) for _ in range(n_images)]
    # split the images over requests, with an empty request in between
    cut = int(rng.integers(0, n_images + 1))
    ipr = [cut, 0, n_images - cut]
    return cfg, tpi, ipr


@pytest.mark.parametrize("seed", range(12))
def test_random_small_encoders_match_oracle(seed):
    cfg, tpi, ipr = _random_case(seed)
    say(f"case random {seed}: {cfg} tiles/image {tpi} images/request {ipr}")
    check_case(cfg, tpi, ipr, wseed=seed, pseed=seed + 50, label=f"random{seed}")


def _plain_cfg(**kw):
    cfg = {"image_size": 42, "patch_size": 14, "channels": 3, "hidden": 64, "heads": 1, "mlp": 128, "layers_local": 1,
           "layers_global": 1, "has_cls": 1, "final_ln": 1, "ln_eps": 1e-6, "proj_layers": 1, "proj_dims": (48,),
           "dtype": "bf16", "token_merge": 1}
    cfg.update(kw)
    return cfg


@pytest.mark.parametrize("dh,heads,dtype", [(8, 4, "bf16"), (16, 3, "bf16"), (32, 2, "bf16"), (40, 2, "bf16"), (56, 1, "bf16"),
                                            (88, 2, "bf16"), (104, 1, "bf16"), (112, 2, "bf16"), (120, 1, "bf16"),
                                            (8, 2, "fp32"), (40, 2, "fp32"), (88, 1, "fp32"), (120, 1, "fp32")])
def test_every_accepted_head_dim_matches_oracle(dh, heads, dtype):
    """Head dims that are stored padded (to 64, 96 or 128 columns per head, zero weight rows) with the true head
    dim in the logit scale: every multiple of 8 the library accepts that the presets and the random cases leave out."""
    cfg = _plain_cfg(hidden=dh * heads, heads=heads, mlp=8 * (dh // 8 + 5), dtype=dtype)
    say(f"case head dim {dh} x {heads} heads, {dtype}")
    check_case(cfg, [2, 1, 3], [1, 0, 2], wseed=dh, pseed=dh + 1, label=f"dh{dh}")


@pytest.mark.parametrize("channels,dtype", [(1, "bf16"), (4, "bf16"), (1, "fp32"), (4, "fp32"), (16, "bf16")])
def test_channel_counts_other_than_three(channels, dtype):
    """Patch vectors of C p^2 values for C = 1, 4 and the maximum, 16 (the patch product's contraction length
    196, 784, 3136 before padding)."""
    cfg = _plain_cfg(channels=channels, dtype=dtype, hidden=128, heads=2)
    say(f"case {channels} channels, {dtype}")
    check_case(cfg, [1, 2], [2], wseed=channels, pseed=7, label=f"C{channels}")


@pytest.mark.parametrize("has_cls,dtype", [(0, "bf16"), (1, "bf16"), (0, "fp32"), (1, "fp32")])
def test_one_patch_tiles(has_cls, dtype):
    """Tiles of a single patch (image side = patch side): one token per tile, or two with the CLS row; local
    attention over one or two keys, global attention over the few tokens of an image."""
    cfg = _plain_cfg(image_size=14, has_cls=has_cls, dtype=dtype, hidden=128, heads=2, layers_local=2)
    assert gen.tokens_per_tile(cfg) == 1 + has_cls
    say(f"case one-patch tiles, has_cls={has_cls}, {dtype}")
    check_case(cfg, [1, 3, 1, 2], [2, 0, 2], wseed=11, pseed=12, label=f"one-patch cls{has_cls}")


@pytest.mark.parametrize("amp", [64.0, 112.0, -112.0])
def test_attention_logits_that_outgrow_the_reference_maximum(amp):
    """Logits that span far more than 2^64 (as exp2 arguments) over the keys of a segment: every query is
    -amp e_0, key t carries 8 cos(pi t / 256) in channel 0 (a position table on a circle, which LayerNorm maps to
    that), so the logit of key t is -amp cos(pi t / 256): -amp ... +amp over 257 keys = five key tiles.
    amp = 64 (+-92 in log2 units) is the most the attention kernel's pass without a reference maximum takes;
    amp = +-112 (+-162 in log2 units, rising resp. falling along the keys) overflows resp. underflows there, so
    the workgroups must notice and run the general pass, whose reference has to move several times after the
    first tile with the accumulated output rescaled each time; a lost rescale or a missed fall-back would show as
    garbage, inf or NaN."""
    cfg = {"image_size": 64, "patch_size": 4, "channels": 3, "hidden": 64, "heads": 1, "mlp": 64, "layers_local": 1,
           "layers_global": 0, "has_cls": 1, "final_ln": 0, "ln_eps": 1e-6, "proj_layers": 0, "proj_dims": (),
           "dtype": "bf16", "token_merge": 1}
    T, D = gen.tokens_per_tile(cfg), 64
    assert T == 257
    w = gen.make_weights(cfg, seed=3).copy()
    off = {}
    o = 0
    for name, shape in gen.weight_layout(cfg):
        n = int(np.prod(shape))
        off[name] = (o, shape)
        o += n

    def view(name):
        a, shape = off[name]
        return w[a:a + int(np.prod(shape))].reshape(shape)

    theta = np.pi * np.arange(T) / (T - 1)
    view("pos")[:, 0] = 4.0 * np.cos(theta)
    view("pos")[:, 1] = 4.0 * np.sin(theta)
    view("l0.ln1_g")[:] = 1.0
    view("l0.ln1_b")[:] = 0.0
    wqkv, bqkv = view("l0.wqkv"), view("l0.bqkv")
    wqkv[:D] = 0.0
    bqkv[:D] = 0.0
    bqkv[0] = -amp                        # q = -amp e_0 for every token
    wqkv[D, :] = 0.0
    wqkv[D, 0] = 1.0                      # k[0] = normalised channel 0 = 8 cos(theta)
    bqkv[D] = 0.0
    wqkv[2 * D:] *= 10.0                  # values and output projection large enough to matter beside x
    view("l0.wo")[:] *= 10.0
    w = gen.round_to_bf16(w)
    px = gen.make_pixels(cfg, 3, seed=5)
    to = np.array([0, 1, 3], dtype=np.int32)
    say(f"case logits outgrowing the softmax reference (257 keys, logits {-amp:+.0f} ... {amp:+.0f})")
    got, _ = gpu_encode(cfg, w, px, [2], to)
    want, _ = O.vit_oracle_encode(cfg, w, px, [2], to)
    assert_parity(got, want, "bf16", f"logits amp {amp:+.0f}")
