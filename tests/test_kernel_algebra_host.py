"""Two facts about fp32 arithmetic that the tuned kernels rely on, checked here with
NumPy float32 (every operation separately rounded, like the kernels and the oracle):

1. With |y| <= s, floor((y + s) * inv + u) never exceeds L, so the clamp of the
   rounding rule is dead whenever s is the chunk's own largest magnitude.
2. For 2^-100 <= s <= 2^100 the normalisation y = v * 2^-7 can be folded into the
   quantizer's constants: (v * 2^-7 + s) * inv == (v + 2^7 s) * (2^-7 inv) bit for bit.
"""
import numpy as np
import pytest

F = np.float32


def _random_scales(rng, count, lo_exp, hi_exp):
    mant = rng.integers(0, 1 << 23, size=count, dtype=np.uint32)
    expo = rng.integers(lo_exp + 127, hi_exp + 127, size=count, dtype=np.uint32)
    return ((expo << np.uint32(23)) | mant).view(F)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_clamp_is_dead_when_scale_is_the_largest_magnitude(bits):
    L = F((1 << bits) - 1)
    rng = np.random.default_rng(5)
    s = _random_scales(rng, 2_000_000, -120, 120)
    two = s + s
    inv = L / two
    u_max = F(255.5 / 256.0)
    # y = s is the worst case (pos is monotone in y); also the few values just below it
    for y in (s, np.nextafter(s, F(0)), s * F(0.999)):
        t = (y + s) * inv + u_max
        assert t.dtype == F
        assert (np.floor(t) <= L).all()
    # and the lower end never goes negative
    assert ((-s + s) * inv >= 0).all()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_folded_normalisation_is_bit_exact_inside_its_range(bits):
    L = F((1 << bits) - 1)
    rng = np.random.default_rng(11)
    count = 2_000_000
    s = _random_scales(rng, count, -100, 100)
    s[:4] = F(2.0) ** F(-100), F(2.0) ** F(100), np.nextafter(F(2.0) ** F(100), F(0)), F(2.0) ** F(-99)
    # v = 128 y with |y| <= s, including values that are tiny next to s and exact +-s
    frac = rng.uniform(-1.0, 1.0, size=count)
    frac[::7] = rng.choice([-1.0, 1.0], size=frac[::7].shape)
    frac[3::11] *= 2.0 ** -30
    y_exact = (s.astype(np.float64) * frac).astype(F)
    y_exact = np.clip(y_exact, -s, s)
    v = y_exact * F(128.0)
    assert np.isfinite(v).all()
    inv = L / (s + s)
    plain = (v * F(0.0078125) + s) * inv
    folded = (v + s * F(128.0)) * (inv * F(0.0078125))
    assert plain.dtype == F and folded.dtype == F
    assert np.array_equal(plain.view(np.uint32), folded.view(np.uint32))
    # tiny v (y underflows to subnormal or zero) changes nothing either
    v_tiny = (rng.uniform(-1, 1, size=count) * 2.0 ** -140).astype(F)
    plain = (v_tiny * F(0.0078125) + s) * inv
    folded = (v_tiny + s * F(128.0)) * (inv * F(0.0078125))
    assert np.array_equal(plain.view(np.uint32), folded.view(np.uint32))
