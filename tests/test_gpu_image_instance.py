"""The pieces around the encoder composed as the paper's Image Instance does (Sec. 4, 4.3): raw images are
preprocessed on the GPU, every image is routed to the instance with the least pending image tokens, each
instance's queue is packed into launches, encoded, published image by image, and the consumer pulls a request
when all of its images are there.  Checked per request against oracle preprocessing + oracle encoding."""
import numpy as np
import pytest

import gen
from oracle import preprocess_oracle as P
from oracle import vit_oracle as O
from parity_util import assert_parity, say

pytestmark = pytest.mark.gpu

MEAN, STD = (0.48, 0.45, 0.41), (0.27, 0.26, 0.28)


def test_image_instance_pipeline_matches_the_oracle_per_request():
    import torch

    import paper_2502_00937_amd as V
    from paper_2502_00937_amd.router import ImageTokenRouter, LaunchPacker

    cfg = gen.get_config("test_merge_bf16")       # 56-px tiles, 2 x 2 token down-sampling: 16 tokens per tile
    S, T_enc, T_out = cfg["image_size"], gen.tokens_per_tile(cfg), gen.out_tokens_per_tile(cfg)
    weights = gen.make_weights(cfg, seed=0)
    # (height, width, tile grid rows, cols) of every raw image of every request; a thumbnail is always added
    requests = {
        10: [(90, 130, 1, 2), (40, 40, 1, 1)],
        11: [],                                    # text-only: never reaches the encoder
        12: [(200, 100, 2, 1), (64, 64, 1, 1), (120, 180, 2, 2)],
        13: [(57, 57, 1, 1)],
    }
    say(f"case image instance pipeline: {sum(len(v) for v in requests.values())} images in {len(requests)} requests")
    raw = {(rid, k): gen.make_image_u8(h, w, 3, seed=100 * rid + k)
           for rid, imgs in requests.items() for k, (h, w, _, _) in enumerate(imgs)}
    tiles_of = {(rid, k): r * c + 1 for rid, imgs in requests.items() for k, (_, _, r, c) in enumerate(imgs)}

    # ---- producer side: preprocess, route, pack, encode, publish
    router = ImageTokenRouter(2, T_enc)
    packers = [LaunchPacker(), LaunchPacker()]
    handoff = V.TokenHandoff(0)
    pixels = {}
    for rid, imgs in requests.items():
        if not imgs:
            continue
        handoff.expect(rid, len(imgs))
        tiles = [tiles_of[(rid, k)] for k in range(len(imgs))]
        for k, inst in enumerate(router.route(tiles)):
            _, _, r, c = imgs[k]
            pixels[(rid, k)] = V.preprocess_tiles(torch.from_numpy(raw[(rid, k)]).cuda(), S, r, c, True, MEAN, STD)
            packers[inst].push(rid, k, tiles[k])
    encoders = [V.VitEncoder(cfg, weights, device=0) for _ in range(2)]   # two instances modelled on the one GPU
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    keep = []                                                            # producer memory lives until release
    torch.cuda.synchronize()
    for inst, p in enumerate(packers):
        with torch.cuda.stream(streams[inst]):
            while len(p):
                items, ipr, to = p.next_launch(max_images=2)
                px = torch.cat([pixels[(i.request_id, i.image_index)] for i in items])
                out, _ = encoders[inst].encode(px, ipr, to)
                keep.append((px, out))
                for j, it in enumerate(items):
                    rows = out[int(to[j]) * T_out:int(to[j + 1]) * T_out]
                    handoff.publish(it.request_id, it.image_index, rows.data_ptr(), rows.numel() * rows.element_size(),
                                    streams[inst].cuda_stream)
                    router.complete(inst, it.tiles)
    assert router.pending == [0, 0]

    # ---- consumer side: pull every complete request on the default stream, compare with the oracle
    wparsed = O.unpack_weights(cfg, weights, np.float64)
    for rid, imgs in requests.items():
        if not imgs:
            continue
        done, nbytes = handoff.complete(rid)
        n_tok = sum(tiles_of[(rid, k)] for k in range(len(imgs))) * T_out
        assert done and nbytes == n_tok * cfg["proj_dims"][-1] * 2
        dst = torch.empty((n_tok, cfg["proj_dims"][-1]), dtype=torch.bfloat16, device="cuda")
        assert handoff.pull(rid, dst.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream) == nbytes
        torch.cuda.synchronize()
        got = dst.float().cpu().numpy()
        want_px = [P.preprocess_tiles(raw[(rid, k)], S, r, c, True, MEAN, STD) for k, (_, _, r, c) in enumerate(imgs)]
        to = np.concatenate([[0], np.cumsum([w.shape[0] for w in want_px])]).astype(np.int32)
        want, _ = O.vit_oracle_encode(cfg, wparsed, np.concatenate(want_px), [len(imgs)], to)
        assert_parity(got, want, "bf16", f"request {rid}")
        handoff.release(rid)
    handoff.close()
    for e in encoders:
        e.close()


def test_real_time_instance_encodes_every_image_once_and_as_if_alone():
    """`ImageInstance.run_stream` on a seeded request stream that arrives faster than single launches drain it,
    so launches of several images form: every image is encoded exactly once, a request's latency is at least
    the duration of the launch that finished it, launches respect the maximum batch, and the tokens of an image
    are bit for bit those of that image encoded alone (an image does not see what it is batched with)."""
    import torch

    import paper_2502_00937_amd as V
    from paper_2502_00937_amd.image_instance import ImageInstance

    cfg = gen.get_config("test_medium_bf16")
    T = gen.tokens_per_tile(cfg)
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    pool = torch.from_numpy(gen.make_pixels(cfg, 24, seed=4)).cuda()
    rng = np.random.default_rng(11)
    arrivals, t = [], 0.0
    for _ in range(40):
        t += float(rng.exponential(0.15))            # ms: much shorter than a launch
        arrivals.append((t, [int(x) for x in rng.integers(1, 4, size=int(rng.integers(1, 5)))]))
    say(f"case real-time instance: {len(arrivals)} requests, {sum(len(a[1]) for a in arrivals)} images")
    index = lambda r, k, tiles: (5 * r + 3 * k) % (24 - tiles + 1)  # noqa: E731
    seen = {}

    def on_launch(items, out, to):
        for j, it in enumerate(items):
            key = (it.request_id, it.image_index)
            assert key not in seen
            seen[key] = out[int(to[j]) * T:int(to[j + 1]) * T].clone()

    inst = ImageInstance(enc, pool, max_images=6, pool_index=index)
    latency, launches = inst.run_stream(arrivals, on_launch)
    assert len(seen) == sum(len(a[1]) for a in arrivals)
    assert all(1 <= n <= 6 for n, _, _ in launches) and max(n for n, _, _ in launches) > 1
    assert sum(n for n, _, _ in launches) == len(seen)
    assert min(latency) >= min(ms for _, _, ms in launches) > 0.0
    say(f"    {len(launches)} launches, up to {max(n for n, _, _ in launches)} images; latency max {max(latency):.2f} ms")
    for (r, k), got in list(seen.items())[::7]:
        tiles = arrivals[r][1][k]
        first = index(r, k, tiles)
        alone, _ = enc.encode(pool[first:first + tiles], [1], np.array([0, tiles], dtype=np.int32))
        torch.cuda.synchronize()
        assert torch.equal(alone.view(torch.int16), got.view(torch.int16)), (r, k)
    enc.close()
