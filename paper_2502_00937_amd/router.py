"""Image-token-load-aware routing and launch packing in front of `vit_encode_packed` (host logic).

Sec. 4.3 of the paper, "Request Routing Across Instances": an image-text request goes to the Image
Instances with the least image-token load, image by image, so a request with many images spreads
over several instances and its images interleave with other requests' (request chunking).  Each
instance then packs what waits in its queue into launches of at most its maximum batch (Sec. 4.2,
"Identifying Max Batch Size").  The image-token count of an image is the static product
tiles * tokens-per-tile (Sec. 4.2), known before any pixel is touched.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass
from typing import Deque, List, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class QueuedImage:
    request_id: int
    image_index: int  # position of the image inside its request
    tiles: int


class ImageTokenRouter:
    """Keeps the pending image-token load of every Image Instance and routes image by image."""

    def __init__(self, n_instances: int, tokens_per_tile: int):
        if n_instances <= 0 or tokens_per_tile <= 0:
            raise ValueError("need at least one instance and a positive token count per tile")
        self.tokens_per_tile = tokens_per_tile
        self.pending = [0] * n_instances  # image tokens queued or running per instance

    def route(self, tiles_per_image: Sequence[int]) -> List[int]:
        """Instance index for every image of one request: each image goes to the instance with the
        least pending image tokens at that moment (ties: lowest index), which then carries its load."""
        if any(t <= 0 for t in tiles_per_image):
            raise ValueError("an image has at least one tile")  # checked first: a bad request changes nothing
        out = []
        for tiles in tiles_per_image:
            i = min(range(len(self.pending)), key=lambda k: (self.pending[k], k))
            self.pending[i] += tiles * self.tokens_per_tile
            out.append(i)
        return out

    def route_whole_request(self, tiles_per_image: Sequence[int], instance: int) -> List[int]:
        """Request-level placement (the baseline the paper argues against): all images on one instance."""
        self.pending[instance] += sum(tiles_per_image) * self.tokens_per_tile
        return [instance] * len(tiles_per_image)

    def complete(self, instance: int, tiles: int) -> None:
        self.pending[instance] -= tiles * self.tokens_per_tile
        if self.pending[instance] < 0:
            raise ValueError("more image tokens completed than were routed to the instance")


class LaunchPacker:
    """FIFO of the images routed to one instance; cuts it into packed launches."""

    def __init__(self):
        self.queue: Deque[QueuedImage] = deque()

    def push(self, request_id: int, image_index: int, tiles: int) -> None:
        self.queue.append(QueuedImage(request_id, image_index, tiles))

    def __len__(self):
        return len(self.queue)

    def next_launch(self, max_images: int, max_tiles: int = 1 << 30) -> Tuple[List[QueuedImage], np.ndarray, np.ndarray]:
        """Pop up to max_images images (and at most max_tiles tiles, but always at least one image) in
        arrival order.  Returns the images, `images_per_request` (consecutive images of one request form
        one packed request) and `tile_offsets` for `vit_encode_packed`."""
        if max_images <= 0:
            raise ValueError("max_images must be positive")
        items: List[QueuedImage] = []
        tiles = 0
        while self.queue and len(items) < max_images and (not items or tiles + self.queue[0].tiles <= max_tiles):
            it = self.queue.popleft()
            items.append(it)
            tiles += it.tiles
        ipr: List[int] = []
        last = None
        for it in items:
            if it.request_id == last:
                ipr[-1] += 1
            else:
                ipr.append(1)
                last = it.request_id
        tile_offsets = np.zeros(len(items) + 1, dtype=np.int32)
        np.cumsum([it.tiles for it in items], out=tile_offsets[1:])
        return items, np.asarray(ipr, dtype=np.int32), tile_offsets


def simulate(arrivals, n_instances: int, tokens_per_tile: int, latency_ms, max_images: int, policy: str):
    """Event-driven model of N Image Instances fed by one router.

    arrivals: list of (time_ms, tiles_per_image list) in time order.
    latency_ms(images, tiles): launch latency of one packed launch (from the measured stage profile).
    policy: "least_image_tokens" (the paper's, image by image) or "round_robin_request" (whole request
    to the next instance in turn).  An instance launches whenever it is idle and its queue is not
    empty, with up to max_images images.  Returns the encode latency per request in ms: last image of
    the request encoded minus arrival.
    """
    router = ImageTokenRouter(n_instances, tokens_per_tile)
    packers = [LaunchPacker() for _ in range(n_instances)]
    busy_until = [0.0] * n_instances
    running: List[List[QueuedImage]] = [[] for _ in range(n_instances)]
    remaining = {}
    arrival_time = {}
    done = {}
    rr = 0

    def start(i: int, now: float):
        items, _, to = packers[i].next_launch(max_images)
        running[i] = items
        busy_until[i] = now + latency_ms(len(items), int(to[-1]))

    def finish(i: int):
        t = busy_until[i]
        for it in running[i]:
            router.complete(i, it.tiles)
            remaining[it.request_id] -= 1
            if remaining[it.request_id] == 0:
                done[it.request_id] = t - arrival_time[it.request_id]
        running[i] = []

    def drain(until: float):
        # complete launches in time order up to `until`; an instance that goes idle starts its next launch
        while True:
            act = [i for i in range(n_instances) if running[i] and busy_until[i] <= until]
            if not act:
                return
            i = min(act, key=lambda k: (busy_until[k], k))
            t = busy_until[i]
            finish(i)
            if len(packers[i]):
                start(i, t)

    for rid, (t, tiles) in enumerate(arrivals):
        drain(t)
        arrival_time[rid] = t
        remaining[rid] = len(tiles)
        if policy == "least_image_tokens":
            where = router.route(tiles)
        elif policy == "round_robin_request":
            where = router.route_whole_request(tiles, rr % n_instances)
            rr += 1
        else:
            raise ValueError(policy)
        for k, (inst, n) in enumerate(zip(where, tiles)):
            packers[inst].push(rid, k, n)
        for i in set(where):
            if not running[i]:
                start(i, t)
    drain(float("inf"))
    return [done[r] for r in range(len(arrivals))]
