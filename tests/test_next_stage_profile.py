"""Host logic of the encoder stage profile (Sec. 4.1, 4.2 of the paper): interpolation, maximum batch under
a latency SLO, capacity MC and ceil(ML / MC), checked against closed forms on synthetic profiles."""
import math

import pytest

from paper_2502_00937_amd import stage_profile as SP
from paper_2502_00937_amd.stage_profile import (ProfilePoint, capacity_tokens_per_s, latency_at,
                                                max_batch_under_slo, replicas)

LINEAR = [ProfilePoint(n, n * 100, 2.0 + 0.5 * n) for n in (1, 4, 16, 64)]  # latency = 2 + n / 2 ms


def test_interpolation_is_exact_at_and_between_the_points_of_a_linear_profile():
    for n in (1, 2, 4, 10, 16, 63, 64, 100, 1000):  # inside and beyond the measured range
        assert latency_at(LINEAR, n) == pytest.approx(2.0 + 0.5 * n)
    assert latency_at(LINEAR, 0.5) == 2.5  # never cheaper than the smallest measured launch


def test_piecewise_profile_uses_the_neighbouring_points_only():
    pts = [ProfilePoint(1, 1, 4.0), ProfilePoint(8, 8, 6.0), ProfilePoint(64, 64, 30.0)]
    assert latency_at(pts, 8) == 6.0
    assert latency_at(pts, 36) == pytest.approx(6.0 + 24.0 * 28 / 56)
    assert latency_at(pts, 120) == pytest.approx(30.0 + 24.0 * 56 / 56)  # last slope continues


def test_max_batch_is_the_closed_form_of_a_linear_latency():
    for slo in (2.4, 2.5, 3.0, 10.0, 34.0, 77.7, 1000.0):
        want = int(math.floor((slo - 2.0) / 0.5)) if slo >= 2.5 else 0
        assert max_batch_under_slo(LINEAR, slo) == want, slo
        if want:
            assert latency_at(LINEAR, want) <= slo < latency_at(LINEAR, want + 1)


def test_capacity_and_replicas_follow_the_paper_formula():
    slo = 34.0  # max batch 64
    mc = capacity_tokens_per_s(LINEAR, slo, tokens_per_image=100)
    assert mc == pytest.approx(64 * 100 / 34e-3)  # throughput grows with the batch on a linear profile
    assert replicas(0.0, mc) == 0
    assert replicas(1.0, mc) == 1
    assert replicas(mc, mc) == 1
    assert replicas(mc * 1.0001, mc) == 2
    assert replicas(mc * 7.5, mc) == 8
    assert capacity_tokens_per_s(LINEAR, 2.0, 100) == 0.0  # even one image misses the SLO
    with pytest.raises(ValueError):
        replicas(10.0, 0.0)


def test_bad_profiles_are_rejected():
    with pytest.raises(ValueError):
        latency_at([], 1)
    with pytest.raises(ValueError):
        latency_at([ProfilePoint(4, 4, 1.0), ProfilePoint(4, 4, 2.0)], 1)
    assert latency_at([ProfilePoint(4, 4, 2.0)], 8) == 4.0  # one point: proportional


def test_profile_round_trips_through_a_file(tmp_path):
    prof = [SP.ProfilePoint(8, 4616, 5.6), SP.ProfilePoint(1, 577, 2.8), SP.ProfilePoint(64, 36928, 30.3)]
    path = tmp_path / "profile.json"
    SP.save_profile(str(path), prof, meta={"encoder": "test", "device": "none"})
    back = SP.load_profile(str(path))
    assert back == sorted(prof, key=lambda p: p.images)
    assert SP.max_batch_under_slo(back, 10.0) == SP.max_batch_under_slo(prof, 10.0)
