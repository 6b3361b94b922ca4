"""The bf16 path's GELU (csrc/common.h: gelu_fast_half, a clamped odd polynomial for erf) against the erf form
the oracle uses.  The coefficients are read out of the header and the function is evaluated here in float32 the
way the kernel evaluates it (Horner with fused multiply-adds is emulated in float64 and rounded per step, which
bounds the kernel's own rounding from above), so the error bound the header states is checked on the CPU."""
import math
import os
import re

import numpy as np

from oracle import vit_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _coefficients():
    src = open(os.path.join(ROOT, "paper_2502_00937_amd", "csrc", "common.h")).read()
    body = src[src.index("float gelu_fast_half(float h)"):]
    body = body[:body.index("return")]
    clamp = float(re.search(r"fminf\(fabsf\(h\), ([0-9.e+-]+)f\)", body).group(1))
    first = re.search(r"float p = fmaf\(([0-9.e+-]+)f, u, ([0-9.e+-]+)f\);", body)
    coeffs = [float(first.group(1)), float(first.group(2))]
    coeffs += [float(c) for c in re.findall(r"p = fmaf\(p, u, ([0-9.e+-]+)f\);", body)]
    return clamp, coeffs  # highest degree first


def _gelu_fast_half(h, clamp, coeffs):
    f32 = np.float32
    h = h.astype(f32)
    t = np.minimum(np.abs(h), f32(clamp))
    u = (t * t).astype(f32)
    p = np.full_like(u, f32(coeffs[0]))
    for c in coeffs[1:]:
        p = (p.astype(np.float64) * u + np.float64(f32(c))).astype(f32)  # one rounding per fused multiply-add
    e = (t * p).astype(f32)
    return (np.abs(h).astype(np.float64) * e + h).astype(f32), e


def test_polynomial_gelu_stays_within_its_stated_error_and_never_overshoots():
    clamp, coeffs = _coefficients()
    assert len(coeffs) == 7 and clamp == 2.0  # degree 6 in t^2, argument halved: |z| clamped at 4
    z = np.linspace(-50.0, 50.0, 2_000_001)
    got, e = _gelu_fast_half(0.5 * z, clamp, coeffs)
    want = O.gelu(z)
    err = np.abs(got.astype(np.float64) - want)
    assert err.max() <= 1.9e-4 + 1e-6, err.max()
    assert 3.5 < abs(z[err.argmax()]) < 4.3            # the largest error sits where bf16 itself steps by 1.6e-2
    assert e.max() < 1.0 and e.min() >= 0.0            # the erf value never reaches 1: no sign flip for z << 0
    big = np.abs(z) >= 8.0
    assert np.all(np.abs(got[big] - np.where(z[big] > 0, z[big], 0.0)) <= 3e-6 * np.abs(z[big]) + 1e-12)
    assert got[z == 0.0][0] == 0.0


def test_polynomial_gelu_against_libm_erf_at_a_few_points():
    clamp, coeffs = _coefficients()
    for zv in (-3.0, -1.0, -0.25, 0.5, 1.0, 2.0, 3.9):
        got, _ = _gelu_fast_half(np.array([0.5 * zv]), clamp, coeffs)
        want = 0.5 * zv * (1.0 + math.erf(zv / math.sqrt(2.0)))
        assert abs(float(got[0]) - want) <= 2e-4, (zv, float(got[0]), want)
