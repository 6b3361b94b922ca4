"""Stage profile on the device (paper Sec. 4.1 "offline profile", Sec. 4.2 "Identifying Max Batch Size" and the
capacity MC of ceil(ML / MC)): measure the profile of the ViT-L/14-336 encoder, take the maximum batch under a
latency SLO, launch exactly that batch and check that it meets the SLO, and compare the capacity the profile
predicts with back-to-back launches."""
import time

import numpy as np
import pytest

import gen
from parity_util import say

pytestmark = pytest.mark.gpu


def _median_launch_ms(torch, enc, px, n, repeats=7):
    ipr, to = np.ones(n, dtype=np.int32), np.arange(n + 1, dtype=np.int32)
    n_tok, out_dim, _, _ = enc.query(n, n)
    out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
    samples = []
    for it in range(repeats + 2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        enc.encode(px[:n], ipr, to, out=out)
        torch.cuda.synchronize()
        if it >= 2:
            samples.append((time.perf_counter() - t0) * 1e3)
    return float(np.median(samples))


def test_measured_profile_max_batch_and_capacity():
    import torch

    import paper_2502_00937_amd as V
    from paper_2502_00937_amd import stage_profile as SP

    cfg = gen.get_config("cfg2_vitl14_336")
    T = gen.tokens_per_tile(cfg)
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        px = torch.from_numpy(gen.make_pixels(cfg, 40, seed=1)).cuda()
        sizes = (1, 4, 8, 16, 32)
        profile = SP.measure_profile(enc, px, 1, T, sizes)
        say("    profile: " + ", ".join(f"{p.images} images {p.latency_ms:.2f} ms" for p in profile))
        assert [p.images for p in profile] == list(sizes)
        assert [p.tokens for p in profile] == [n * T for n in sizes]
        lat = [p.latency_ms for p in profile]
        assert all(l > 0 for l in lat)
        assert all(b >= 0.95 * a for a, b in zip(lat, lat[1:])), lat       # non-decreasing up to timing noise
        assert lat[-1] > 2.0 * lat[0]                                       # the batch does cost something

        # an SLO between the 16- and the 32-image points: the maximum batch lies strictly between them
        slo = 0.5 * (lat[3] + lat[4])
        b = SP.max_batch_under_slo(profile, slo)
        assert 16 < b < 32, (b, slo)
        assert SP.latency_at(profile, b) <= slo < SP.latency_at(profile, b + 1)
        got = _median_launch_ms(torch, enc, px, b)
        over = _median_launch_ms(torch, enc, px, 32)
        say(f"    SLO {slo:.2f} ms -> max batch {b}: launch of {b} images {got:.2f} ms "
            f"(profile {SP.latency_at(profile, b):.2f}); 32 images {over:.2f} ms")
        assert got <= slo * 1.05, (got, slo)                                # the chosen batch meets the SLO
        assert over > slo                                                   # and a measured larger one does not
        assert abs(got - SP.latency_at(profile, b)) <= 0.10 * got           # interpolation is close to the truth

        # capacity MC: back-to-back launches of the best batch within the SLO
        mc = SP.capacity_tokens_per_s(profile, slo, T)
        ipr, to = np.ones(b, dtype=np.int32), np.arange(b + 1, dtype=np.int32)
        n_tok, out_dim, _, _ = enc.query(b, b)
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        for _ in range(2):
            enc.encode(px[:b], ipr, to, out=out)
        torch.cuda.synchronize()
        launches = 20
        t0 = time.perf_counter()
        for _ in range(launches):
            enc.encode(px[:b], ipr, to, out=out)
        torch.cuda.synchronize()
        measured = launches * b * T / (time.perf_counter() - t0)
        say(f"    capacity: profile {mc / 1e6:.3f} M tokens/s, {launches} back-to-back launches {measured / 1e6:.3f} M tokens/s")
        assert 0.9 * mc <= measured <= 1.25 * mc, (mc, measured)
        assert SP.replicas(5.0 * mc, mc) == 5 and SP.replicas(5.01 * mc, mc) == 6
    finally:
        enc.close()
