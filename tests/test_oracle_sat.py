"""Pins for the oracle of the saturation-based aggregation variant (CPU only): the
operator's definition enumerated, hand-computed order cases, closed forms for the
cases where saturation reduces to something simpler."""
import itertools

import numpy as np
import pytest

from oracle import thc as T
from oracle.thc_sat import sat, sat_aggregate, sat_decode, sat_max, sat_pipeline, sat_quantize


def test_sat_max_values():
    assert [sat_max(b) for b in (2, 4, 8)] == [1, 7, 127]


@pytest.mark.parametrize("bits", [2, 4])
def test_sat_matches_the_printed_formula_on_every_pair(bits):
    M = (1 << (bits - 1)) - 1
    for x, y in itertools.product(range(-M, M + 1), repeat=2):
        want = min(2 ** (bits - 1) - 1, max(-2 ** (bits - 1) + 1, x + y))   # the paper's formula, in Python ints
        got = int(sat(x, y, bits))
        assert got == want
        assert -M <= got <= M
        assert got == int(sat(y, x, bits))          # commutative
    assert int(sat(5 if bits == 4 else 1, 0, bits)) == (5 if bits == 4 else 1)


def test_sat_literal_values_b4():
    assert int(sat(7, 1, 4)) == 7
    assert int(sat(-7, -1, 4)) == -7
    assert int(sat(3, 4, 4)) == 7
    assert int(sat(3, -5, 4)) == -2
    assert int(sat(-6, -6, 4)) == -7


def _payloads_from_z(zs, bits):
    M = sat_max(bits)
    return [T.pack(np.asarray(z, dtype=np.int64) + M, bits) for z in zs]


def test_aggregation_order_is_worker_order():
    """Sat is not associative: 7, 7, -7 gives 0 left to right (7+7 clips to 7, then
    7-7), but 7 right to left.  The oracle takes worker order 0, 1, 2."""
    bits, M = 4, 7
    zs = [[7, -7, 7, 1], [7, 7, -7, 2], [-7, 7, 7, 3]]
    A, clipped = sat_aggregate(_payloads_from_z(zs, bits), bits, count=4)
    assert (A.astype(int) - M).tolist() == [0, 7, 7, 6]
    assert clipped.tolist() == [True, False, False, False]
    # the other association of the first column, by hand: Sat(7, Sat(7, -7)) = 7
    assert int(sat(7, sat(7, -7, bits), bits)) == 7


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_same_sign_values_saturate_to_the_clamped_sum(bits):
    """When every worker's value has the same sign the running Sat equals the clamp of
    the exact sum (closed form)."""
    M = sat_max(bits)
    rng = np.random.default_rng(bits)
    W, n = 6, 4096
    z = rng.integers(0, M + 1, size=(W, n))
    z[:, n // 2:] *= -1
    A, clipped = sat_aggregate(_payloads_from_z(z, bits), bits)
    exact = z.sum(axis=0)
    assert ((A.astype(int) - M) == np.clip(exact, -M, M)).all()
    assert (clipped == (np.abs(exact) > M)).all()


@pytest.mark.parametrize("bits", [4, 8])
def test_without_clipping_it_is_the_exact_sum_and_decodes_like_the_exact_path(bits):
    M = sat_max(bits)
    rng = np.random.default_rng(3)
    W, log2c = 4, 6
    c = 1 << log2c
    n = 5 * c
    z = rng.integers(-(M // W), M // W + 1, size=(W, n))      # prefix sums stay inside [-M, M]
    pay = _payloads_from_z(z, bits)
    A, clipped = sat_aggregate(pay, bits)
    assert not clipped.any()
    assert ((A.astype(int) - M) == z.sum(axis=0)).all()
    # decode: (sum of idx) * step / W - s  with  sum of idx = A - M + W M  and  M step = s
    scale = rng.uniform(0.1, 2.0, size=n // c)
    got = sat_decode(A, scale, W, n, log2c, 9, bits)
    S = (z + M).sum(axis=0).reshape(-1, c)
    s = scale.reshape(-1, 1)
    yhat = S * ((s + s) / (2 * M) / W) - s
    want = T.rht_inverse(yhat.reshape(-1), n, log2c, 9)
    assert np.allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_grid_has_zero_and_both_ends_for_every_random_value(bits, dtype):
    M = sat_max(bits)
    log2c = 8
    c = 1 << log2c
    s = np.array([0.37], dtype=dtype)
    for r in range(256):
        rr = np.full(c, r)
        assert (sat_quantize(np.zeros(c), s, log2c, 0, 1, bits, dtype=dtype, r=rr) == M).all()
        assert (sat_quantize(np.full(c, s[0]), s, log2c, 0, 1, bits, dtype=dtype, r=rr) == 2 * M).all()
        assert (sat_quantize(np.full(c, -s[0]), s, log2c, 0, 1, bits, dtype=dtype, r=rr) == 0).all()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_scale_too_small_for_the_reciprocal_step_gives_the_centre(dtype):
    """Below 2 s = 2^-119 the chunk is quantized like an all-zero one: the centre index (z = 0);
    at that value the ordinary rule applies, ends included."""
    bits, M, c = 8, sat_max(8), 8
    frac = np.array([1.0, -1.0, 0.0, 0.3, -0.7, 0.9, -0.2, 0.5])
    for two_s, empty in ((2.0 ** -120, True), (2.0 ** -119, False)):
        s = np.array([two_s / 2], dtype=dtype)
        y = (frac * float(s[0])).astype(dtype)
        with np.errstate(all="raise"):
            idx = sat_quantize(y, s, 3, 0, 1, bits, dtype=dtype)
        if empty:
            assert (idx == M).all()
        else:
            assert idx[0] == 2 * M and idx[1] == 0 and idx[2] == M


def test_rounding_probability_is_the_fraction_brute_force():
    bits, log2c = 4, 3
    M, c = 7, 8
    s = np.array([1.0])
    y = np.linspace(-0.9, 0.9, c)
    v = (y + 1.0) * (2 * M / 2.0)
    ups = np.zeros(c)
    for r in range(256):
        idx = sat_quantize(y, s, log2c, 0, 0, bits, r=np.full(c, r))
        ups += idx == np.floor(v) + 1
    want = np.array([sum(1 for r in range(256) if (r + 0.5) / 256 >= 1 - (x - np.floor(x))) for x in v])
    assert (ups == want).all()


def test_single_worker_round_trip_within_one_step_and_exact_on_grid():
    bits, log2c, seed = 4, 7, 5
    M, c = 7, 128
    rng = np.random.default_rng(0)
    x = rng.normal(size=3 * c).astype(np.float32)
    res = sat_pipeline([x], log2c, seed, bits)
    assert not res["clipped"].any()
    assert (res["aggregate"] == res["idx"][0]).all()          # W = 1: nothing to add
    y = res["y"][0].reshape(-1, c)
    step = (2 * res["scale"] / (2 * M)).reshape(-1, 1)
    yhat = (res["aggregate"].astype(float).reshape(-1, c) - M) * step
    assert (np.abs(yhat - y) < step).all()
    assert res["packed_aggregate"].dtype == np.uint8
    assert (T.unpack(res["packed_aggregate"], bits) <= 2 * M).all()   # all-ones code never occurs


def test_clipping_grows_with_the_number_of_workers():
    """Independent workers: the paper notes that more workers mean more overflow at
    fixed b.  Same data prefix for every W, so the rates are nested."""
    bits, log2c, seed = 4, 10, 2
    rng = np.random.default_rng(1)
    xs = [rng.normal(size=1 << 12).astype(np.float32) for _ in range(16)]
    rates = []
    for W in (2, 4, 8, 16):
        res = sat_pipeline(xs[:W], log2c, seed, bits)
        assert (np.abs(res["aggregate"].astype(int) - 7) <= 7).all()
        rates.append(res["clipped"].mean())
    assert rates[0] < rates[1] < rates[2] < rates[3]
    assert rates[0] < 0.01


def test_fp32_mode_agrees_with_the_definition():
    bits, log2c, seed = 4, 9, 11
    rng = np.random.default_rng(4)
    xs = [(rng.standard_t(3, size=2000) * 1e-3).astype(np.float32) for _ in range(4)]
    r64 = sat_pipeline(xs, log2c, seed, bits, dtype=np.float64)
    r32 = sat_pipeline(xs, log2c, seed, bits, dtype=np.float32)
    mism = sum(int((a != b).sum()) for a, b in zip(r64["idx"], r32["idx"]))
    assert mism <= 2                                   # only values within rounding of a grid boundary
    if mism == 0:
        err = np.linalg.norm(r32["out"] - r64["out"]) / np.linalg.norm(r64["out"])
        assert err < 1e-5
