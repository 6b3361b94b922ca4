"""Host logic of image-token-load-aware routing and launch packing (Sec. 4.3 of the paper)."""
import numpy as np
import pytest

from paper_2502_00937_amd.router import ImageTokenRouter, LaunchPacker, simulate


def naive_route(pending, tiles_per_image, tokens_per_tile):
    """Independent restatement of the rule: every image to the currently least loaded instance."""
    pending = list(pending)
    out = []
    for t in tiles_per_image:
        best = 0
        for k in range(1, len(pending)):
            if pending[k] < pending[best]:
                best = k
        pending[best] += t * tokens_per_tile
        out.append(best)
    return out, pending


def test_router_matches_the_rule_on_random_streams_and_conserves_load():
    rng = np.random.default_rng(3)
    r = ImageTokenRouter(5, 577)
    shadow = [0] * 5
    total = 0
    for _ in range(300):
        tiles = [int(x) for x in rng.integers(1, 8, size=int(rng.integers(1, 12)))]
        want, shadow = naive_route(shadow, tiles, 577)
        assert r.route(tiles) == want
        total += sum(tiles) * 577
        assert r.pending == shadow and sum(r.pending) == total
        if rng.random() < 0.5:  # some work finishes
            i = int(np.argmax(r.pending))
            r.complete(i, 1)
            shadow[i] -= 577
            total -= 577


def test_large_request_spreads_over_idle_instances():
    r = ImageTokenRouter(4, 100)
    assert sorted(r.route([1] * 8)) == [0, 0, 1, 1, 2, 2, 3, 3]  # request chunking across instances
    assert r.pending == [200] * 4
    r2 = ImageTokenRouter(3, 10)
    r2.pending = [50, 0, 20]
    assert r2.route([1, 1, 1, 1]) == [1, 1, 1, 2]  # ties go to the lowest index


def test_router_rejects_bad_input():
    with pytest.raises(ValueError):
        ImageTokenRouter(0, 1)
    r = ImageTokenRouter(2, 10)
    with pytest.raises(ValueError):
        r.route([1, 0])
    assert r.pending == [0, 0]  # a rejected request leaves the loads untouched
    with pytest.raises(ValueError):
        r.complete(0, 1)


def test_packer_builds_valid_packed_launches():
    p = LaunchPacker()
    for rid, tiles in [(7, [2, 1]), (8, [3]), (7, [1]), (9, [1, 1, 4])]:  # request 7 comes back after 8
        for k, t in enumerate(tiles):
            p.push(rid, k, t)
    items, ipr, to = p.next_launch(max_images=5)
    assert [(i.request_id, i.tiles) for i in items] == [(7, 2), (7, 1), (8, 3), (7, 1), (9, 1)]
    assert ipr.tolist() == [2, 1, 1, 1] and int(ipr.sum()) == len(items)  # non-adjacent images of 7 stay separate
    assert to.tolist() == [0, 2, 3, 6, 7, 8] and to.dtype == np.int32
    items, ipr, to = p.next_launch(max_images=8, max_tiles=4)
    assert [(i.request_id, i.tiles) for i in items] == [(9, 1)] and to.tolist() == [0, 1]  # the 4-tile image waits
    items, ipr, to = p.next_launch(max_images=8, max_tiles=2)
    assert [(i.request_id, i.tiles) for i in items] == [(9, 4)]  # a launch always takes at least one image
    assert len(p) == 0 and p.next_launch(4)[1].size == 0


def test_simulation_one_instance_is_policy_independent_and_fifo():
    arrivals = [(0.0, [1, 1]), (1.0, [1]), (2.0, [1, 1, 1])]
    lat = lambda images, tiles: 10.0 * images  # noqa: E731
    a = simulate(arrivals, 1, 100, lat, 2, "least_image_tokens")
    b = simulate(arrivals, 1, 100, lat, 2, "round_robin_request")
    # launches: [r0,r0] 0-20, [r1,r2] 20-40, [r2,r2] 40-60
    assert a == b == [20.0, 39.0, 58.0]


def test_image_level_routing_cuts_the_tail_of_a_burst():
    # one request with 16 images between single-image requests, 4 instances, latency linear in images
    arrivals = [(0.0, [1] * 16)] + [(0.1 * k, [1]) for k in range(1, 9)]
    lat = lambda images, tiles: 2.0 + 1.0 * images  # noqa: E731
    img = simulate(arrivals, 4, 100, lat, 4, "least_image_tokens")
    req = simulate(arrivals, 4, 100, lat, 4, "round_robin_request")
    assert img[0] < req[0]          # the big request finishes earlier when its images run in parallel
    assert max(img) < max(req)      # and nobody waits behind it for 16 images on one instance
    assert len(img) == len(arrivals) and all(x > 0 for x in img)


def test_percentiles_are_order_statistics():
    from paper_2502_00937_amd.image_instance import percentiles

    v = list(range(1, 101))                        # 1 ... 100: the q-th percentile is q
    assert percentiles(v) == [50.0, 90.0, 99.0]
    assert percentiles([7.0]) == [7.0, 7.0, 7.0]
    assert percentiles([3.0, 1.0, 2.0], qs=(34, 100)) == [2.0, 3.0]
