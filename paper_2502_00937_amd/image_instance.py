"""One Image Instance driven in real time (host loop around the HIP encoder).

Sec. 4 of the paper: an Image Instance takes the images routed to it, batches what waits in its queue
up to the profiled maximum batch (Sec. 4.2, "Identifying Max Batch Size") and encodes batch after
batch; a request's encode latency ends when the last of its images has been encoded.  This module
runs that loop against the wall clock on the one GPU present, so that the event model in `router.py`
(which predicts the same quantity from a stage profile, for any number of instances) can be checked
against real launches for one instance.
"""
from __future__ import annotations

import time
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from .router import LaunchPacker, QueuedImage


class ImageInstance:
    """An encoder, a FIFO of routed images and a pool of device-resident tiles to encode.

    `pixel_pool` is a device tensor [n_pool_tiles, C, S, S].  With `pool_index(request, image, tiles)` given,
    an image reads the pool tiles starting at that row, so that what was encoded can be reproduced (the
    launch's tiles are then gathered into one tensor first); without it a launch reads the first tiles
    of the pool, which is all a timing run needs.
    """

    def __init__(self, enc, pixel_pool, max_images: int, max_tiles: int = 1 << 30,
                 pool_index: Optional[Callable[[int, int, int], int]] = None):
        if max_images <= 0:
            raise ValueError("max_images must be positive")
        self.enc = enc
        self.pool = pixel_pool
        self.max_images = max_images
        self.max_tiles = min(max_tiles, int(pixel_pool.shape[0]))
        self.packer = LaunchPacker()
        self._pool_index = pool_index

    def tile_rows(self, items: Sequence[QueuedImage]):
        """Pool rows of the tiles of a launch, in launch order (needs `pool_index`)."""
        rows = []
        for it in items:
            first = self._pool_index(it.request_id, it.image_index, it.tiles)
            rows.extend(range(first, first + it.tiles))
        return rows

    def run_stream(self, arrivals: Sequence[Tuple[float, Sequence[int]]],
                   on_launch: Optional[Callable] = None) -> Tuple[List[float], List[Tuple[int, int, float]]]:
        """Feed `arrivals` ((time in ms, tiles per image) in time order) to the instance in real time.

        A launch starts as soon as the instance is idle and at least one image waits; it takes what has
        arrived by then, up to the maximum batch.  Returns the encode latency of every request in ms
        (last image encoded minus arrival) and the launch log [(images, tiles, ms)].  `on_launch(items,
        out, tile_offsets)` is called after each launch has finished, with the launch's output tensor.
        """
        import torch

        n = len(arrivals)
        if any(len(t) == 0 or any(x <= 0 for x in t) for _, t in arrivals):
            raise ValueError("every request of the stream needs at least one image and every image a tile")
        if any(x > self.max_tiles for _, t in arrivals for x in t):
            raise ValueError("an image has more tiles than the pixel pool or the launch limit holds")
        remaining = [len(t) for _, t in arrivals]
        latency = [0.0] * n
        launches: List[Tuple[int, int, float]] = []
        dev = self.pool.device
        out_dtype = torch.bfloat16 if self.enc.cfg["dtype"] == "bf16" else torch.float32
        nxt = 0
        done = 0
        torch.cuda.synchronize(dev)
        t0 = time.perf_counter()
        while done < n:
            now = (time.perf_counter() - t0) * 1e3
            while nxt < n and arrivals[nxt][0] <= now:  # admit what has arrived
                for k, tiles in enumerate(arrivals[nxt][1]):
                    self.packer.push(nxt, k, int(tiles))
                nxt += 1
            if not len(self.packer):  # idle: wait for the next arrival
                wait_ms = arrivals[nxt][0] - now
                if wait_ms > 0.3:
                    time.sleep((wait_ms - 0.2) * 1e-3)
                continue
            items, ipr, to = self.packer.next_launch(self.max_images, self.max_tiles)
            if self._pool_index is None:
                px = self.pool[:int(to[-1])]
            else:
                px = self.pool[torch.as_tensor(self.tile_rows(items), device=dev)]
            n_tok, out_dim, _, _ = self.enc.query(int(to[-1]), len(items))
            out = torch.empty((n_tok, out_dim), dtype=out_dtype, device=dev)
            self.enc.encode(px, ipr, to, out=out)
            torch.cuda.synchronize(dev)
            t_done = (time.perf_counter() - t0) * 1e3
            launches.append((len(items), int(to[-1]), t_done - now))
            for it in items:
                remaining[it.request_id] -= 1
                if remaining[it.request_id] == 0:
                    latency[it.request_id] = t_done - arrivals[it.request_id][0]
                    done += 1
            if on_launch is not None:
                on_launch(items, out, to)
        return latency, launches


def percentiles(values: Sequence[float], qs=(50, 90, 99)) -> List[float]:
    v = np.sort(np.asarray(values, dtype=np.float64))
    return [float(v[min(len(v) - 1, int(np.ceil(q / 100.0 * len(v))) - 1)]) for q in qs]
