"""Encoder stage profile, maximum batch size and capacity (host logic around the HIP encoder).

Follows the paper's offline profile generation (Sec. 4.1: profile a set of load levels, extrapolate
in between), "Identifying Max Batch Size" and "Token-Aware Pool Autoscaling" (Sec. 4.2: the number of
replicas of a stage is ceil(ML / MC), ML = modality load in image tokens per second, MC = the most a
replica sustains without violating the latency SLO).  The measurements come from `VitEncoder.encode`;
everything else here is arithmetic on the measured points.
"""
from __future__ import annotations

import math
import time
from dataclasses import dataclass
from typing import Iterable, List, Sequence


@dataclass(frozen=True)
class ProfilePoint:
    images: int        # images in one launch
    tokens: int        # encoder tokens of that launch
    latency_ms: float  # median wall time of one launch, pixels resident in HBM


def measure_profile(enc, pixels, tiles_per_image: int, tokens_per_tile: int, batch_sizes: Iterable[int],
                    repeats: int = 5, warmup: int = 2) -> List[ProfilePoint]:
    """Encode the first n images of `pixels` ([n_tiles, C, S, S], device) for every n in batch_sizes,
    each image a request of its own, and return the median launch latency per size."""
    import numpy as np
    import torch

    points = []
    for n in sorted(set(int(b) for b in batch_sizes)):
        n_tiles = n * tiles_per_image
        if n <= 0 or n_tiles > pixels.shape[0]:
            raise ValueError(f"batch size {n} does not fit the {pixels.shape[0]} tiles provided")
        ipr = np.ones(n, dtype=np.int32)
        to = np.arange(n + 1, dtype=np.int32) * tiles_per_image
        n_tok, out_dim, _, _ = enc.query(n_tiles, n)
        out = torch.empty((n_tok, out_dim), device=pixels.device,
                          dtype=torch.bfloat16 if enc.cfg["dtype"] == "bf16" else torch.float32)
        samples = []
        for it in range(warmup + repeats):
            torch.cuda.synchronize(pixels.device)
            t0 = time.perf_counter()
            enc.encode(pixels[:n_tiles], ipr, to, out=out)
            torch.cuda.synchronize(pixels.device)
            if it >= warmup:
                samples.append((time.perf_counter() - t0) * 1e3)
        samples.sort()
        points.append(ProfilePoint(n, n_tiles * tokens_per_tile, samples[len(samples) // 2]))
    return points


def save_profile(path: str, profile: Sequence[ProfilePoint], meta: dict | None = None) -> None:
    """Write a measured profile as JSON so that it can be cached and shared between instances of the same
    encoder and device type (Sec. 4.1: profiles are generated offline and reused)."""
    import json

    with open(path, "w") as f:
        json.dump({"meta": meta or {}, "points": [[p.images, p.tokens, p.latency_ms] for p in _check(profile)]}, f)


def load_profile(path: str) -> List[ProfilePoint]:
    import json

    with open(path) as f:
        doc = json.load(f)
    return _check([ProfilePoint(int(i), int(t), float(ms)) for i, t, ms in doc["points"]])


def _check(profile: Sequence[ProfilePoint]) -> List[ProfilePoint]:
    pts = sorted(profile, key=lambda p: p.images)
    if not pts:
        raise ValueError("empty profile")
    for a, b in zip(pts, pts[1:]):
        if a.images == b.images:
            raise ValueError("duplicate batch size in profile")
    return pts


def latency_at(profile: Sequence[ProfilePoint], images: float) -> float:
    """Launch latency of a batch of `images`, piecewise linear through the measured points; below the
    first point the first latency (a launch never gets cheaper than the smallest one measured), beyond
    the last point the last segment's slope (encode time grows linearly with the batch, Sec. 3.2)."""
    pts = _check(profile)
    if images <= pts[0].images or len(pts) == 1:
        if len(pts) == 1 and images > pts[0].images:  # one point: latency proportional to the batch
            return pts[0].latency_ms * images / pts[0].images
        return pts[0].latency_ms
    for a, b in zip(pts, pts[1:]):
        if images <= b.images:
            return a.latency_ms + (b.latency_ms - a.latency_ms) * (images - a.images) / (b.images - a.images)
    a, b = pts[-2], pts[-1]
    return b.latency_ms + (b.latency_ms - a.latency_ms) * (images - b.images) / (b.images - a.images)


def max_batch_under_slo(profile: Sequence[ProfilePoint], slo_ms: float, limit: int = 1 << 20) -> int:
    """Largest number of images per launch whose predicted latency stays within the SLO (0 if even the
    smallest measured launch misses it).  Latency is non-decreasing in the batch for a sane profile;
    the search does not assume it and returns the largest batch below the first violation."""
    pts = _check(profile)
    if latency_at(pts, pts[0].images) > slo_ms:
        return 0
    lo, hi = pts[0].images, pts[0].images
    while hi < limit and latency_at(pts, hi * 2) <= slo_ms:  # gallop, then bisect
        hi *= 2
    lo, hi = hi, min(hi * 2, limit)
    if latency_at(pts, hi) <= slo_ms:
        return hi
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if latency_at(pts, mid) <= slo_ms:
            lo = mid
        else:
            hi = mid
    return lo


def capacity_tokens_per_s(profile: Sequence[ProfilePoint], slo_ms: float, tokens_per_image: int) -> float:
    """MC: image tokens per second one replica sustains with back-to-back launches of the best batch
    size that still meets the SLO."""
    b_max = max_batch_under_slo(profile, slo_ms)
    # on every linear piece of the latency curve b / latency(b) is monotone: only the measured sizes
    # up to b_max and b_max itself can be the best
    candidates = sorted({p.images for p in profile if p.images <= b_max} | ({b_max} if b_max > 0 else set()))
    return max((b * tokens_per_image / (latency_at(profile, b) * 1e-3) for b in candidates), default=0.0)


def replicas(load_tokens_per_s: float, capacity_tokens_per_s_: float) -> int:
    """ceil(ML / MC) (Sec. 4.2); at least one replica while there is any load."""
    if load_tokens_per_s <= 0:
        return 0
    if capacity_tokens_per_s_ <= 0:
        raise ValueError("the stage cannot meet the SLO at any batch size: capacity is zero")
    return max(1, math.ceil(load_tokens_per_s / capacity_tokens_per_s_))
