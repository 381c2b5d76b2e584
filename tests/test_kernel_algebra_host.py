"""Two facts about fp32 arithmetic that the tuned kernels rely on, checked here with the
oracle's exact float32 fused multiply-add (tests only; the kernels share no code with it):

1. With |y| <= s the rounding rule's t = fma(y, inv, L/2 + u) (grids of up to 32 points)
   or t = fma(y + s, inv, u) (larger grids) satisfies 0 <= t < L + 1, so the clamp
   min(floor(t), L) is dead whenever s is at least the chunk's own largest magnitude.
   The same on the min/max grid, t = fma(y - lo, inv, u) with inv = L / (hi - lo), when lo
   and hi are the chunk's own extremes.
2. For 2^-100 <= s <= 2^100 the normalisation y = v * 2^-7 can be folded into the
   multiplier: fma(v * 2^-7, inv, c) == fma(v, 2^-7 inv, c) bit for bit, and likewise
   fma(v * 2^-7 + s, inv, u) == fma(v + 128 s, 2^-7 inv, u).
"""
import numpy as np
import pytest

from oracle.thc import fma32

F = np.float32


def _random_scales(rng, count, lo_exp, hi_exp):
    mant = rng.integers(0, 1 << 23, size=count, dtype=np.uint32)
    expo = rng.integers(lo_exp + 127, hi_exp + 127, size=count, dtype=np.uint32)
    return ((expo << np.uint32(23)) | mant).view(F)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_clamp_is_dead_when_scale_is_the_largest_magnitude(bits):
    L = F((1 << bits) - 1)
    half = F(0.5) * L
    rng = np.random.default_rng(5)
    s = _random_scales(rng, 1_000_000, -120, 120)
    inv = L / (s + s)
    c_max = half + F(255.5 / 256.0)
    c_min = half + F(0.5 / 256.0)
    # t is monotone in y: the extremes are y = +s with the largest noise, y = -s with the smallest
    offset = L > 31
    u_max, u_min = F(255.5 / 256.0), F(0.5 / 256.0)
    for y in (s, np.nextafter(s, F(0)), s * F(0.999)):
        t = fma32(y + s, inv, u_max) if offset else fma32(y, inv, c_max)
        assert t.dtype == F
        assert (np.floor(t) <= L).all()
    for y in (-s, -np.nextafter(s, F(0))):
        t = fma32(y + s, inv, u_min) if offset else fma32(y, inv, c_min)
        assert (t > 0).all()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_clamp_is_dead_on_the_min_max_grid_when_the_range_is_the_chunks_own(bits):
    """t = fma(fl(y - lo), inv, u) with inv = fl(L / fl(hi - lo)) and lo <= y <= hi: t is
    monotone in y, so y = hi with the largest noise is the extreme, and floor(t) <= L; at
    y = lo, t = u > 0.  Ranges of every size and position, also lo and hi of opposite sign,
    nearly equal, and hugely different in magnitude; widths from 2^-119 up (below that the
    range is treated as empty, because L / width overflows: 255 / 2^-121 > 2^128)."""
    L = F((1 << bits) - 1)
    rng = np.random.default_rng(17)
    count = 1_000_000
    a = _random_scales(rng, count, -110, 110) * rng.choice([F(-1), F(1)], size=count).astype(F)
    b = _random_scales(rng, count, -110, 110) * rng.choice([F(-1), F(1)], size=count).astype(F)
    b[::5] = a[::5] * (F(1) + F(2.0) ** F(-20))                   # nearly equal
    b[1::5] = np.nextafter(a[1::5], F(np.inf))                     # adjacent floats
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    keep = (hi - lo) >= F(2.0 ** -119)      # narrower ranges are sent as constant chunks (inv = 0)
    lo, hi = lo[keep], hi[keep]
    width = hi - lo
    assert width.dtype == F and len(width) > 500_000
    inv = L / width
    u_max, u_min = F(255.5 / 256.0), F(0.5 / 256.0)
    for y in (hi, np.nextafter(hi, F(-np.inf)), lo + width * F(0.999)):
        y = np.clip(y, lo, hi)
        t = fma32(y - lo, inv, u_max)
        assert t.dtype == F
        assert (np.floor(t) <= L).all()
    assert (fma32(lo - lo, inv, u_min) > 0).all()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_folded_normalisation_is_bit_exact_inside_its_range(bits):
    L = F((1 << bits) - 1)
    rng = np.random.default_rng(11)
    count = 1_000_000
    s = _random_scales(rng, count, -100, 100)
    s[:4] = F(2.0) ** F(-100), F(2.0) ** F(100), np.nextafter(F(2.0) ** F(100), F(0)), F(2.0) ** F(-99)
    # v = 128 y with |y| <= s, including values that are tiny next to s and exact +-s
    frac = rng.uniform(-1.0, 1.0, size=count)
    frac[::7] = rng.choice([-1.0, 1.0], size=frac[::7].shape)
    frac[3::11] *= 2.0 ** -30
    y = np.clip((s.astype(np.float64) * frac).astype(F), -s, s)
    v = y * F(128.0)
    assert np.isfinite(v).all()
    inv = L / (s + s)
    c = F(0.5) * L + ((rng.integers(0, 256, size=count).astype(F) + F(0.5)) * F(2.0 ** -8))
    plain = fma32(v * F(0.0078125), inv, c)
    folded = fma32(v, inv * F(0.0078125), c)
    assert np.array_equal(plain.view(np.uint32), folded.view(np.uint32))
    # the offset form of the large grids: v * 2^-7 + s against (v + 128 s) * 2^-7
    u = c - F(0.5) * L
    plain = fma32(v * F(0.0078125) + s, inv, u)
    folded = fma32(v - F(-128.0) * s, inv * F(0.0078125), u)
    assert np.array_equal(plain.view(np.uint32), folded.view(np.uint32))
    # tiny v (y underflows to subnormal or zero) changes nothing either
    v_tiny = (rng.uniform(-1, 1, size=count) * 2.0 ** -140).astype(F)
    plain = fma32(v_tiny * F(0.0078125), inv, c)
    folded = fma32(v_tiny, inv * F(0.0078125), c)
    assert np.array_equal(plain.view(np.uint32), folded.view(np.uint32))
