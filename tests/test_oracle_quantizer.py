"""Pins for the oracle's quantizer, packing, aggregation and decode (CPU only):
closed forms, brute force over every random value, invariants."""
from fractions import Fraction

import numpy as np
import pytest

from oracle.thc import (RBITS, aggregate, chunk_absmax, decode, pack, pipeline, quantize,
                        rht_forward, rounding_fields, scale_reduce, sum_dtype, unpack)


# ----------------------------------------------------------------------- quantizer
@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_range_ends_map_to_0_and_L_for_every_random_value(bits, dtype):
    L = (1 << bits) - 1
    log2c = 12
    c = 1 << log2c
    s = np.array([0.37, 1e-5], dtype=dtype)
    r = rounding_fields(0, 2 * c, 0, 1)
    assert set(r.tolist()) == set(range(1 << RBITS))          # every r occurs
    top = np.repeat(s, c)
    assert (quantize(top, s, log2c, 0, 1, bits, dtype=dtype) == L).all()
    assert (quantize(-top, s, log2c, 0, 1, bits, dtype=dtype) == 0).all()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_grid_points_are_reproduced_for_every_seed(bits):
    L = (1 << bits) - 1
    log2c = 8
    c = 1 << log2c
    s = L / 2.0                                  # step = 1 exactly
    k = np.arange(c) % (L + 1)
    y = k - s
    for seed in range(20):
        for dtype in (np.float64, np.float32):
            assert (quantize(y, [s], log2c, 3, seed, bits, dtype=dtype) == k).all()


@pytest.mark.parametrize("rbits", [8, 16])
def test_brute_force_rounding_probability(rbits):
    """c = 4 and 8, b = 2: enumerate every r.  The count of r that round up is
    fixed by exact rational arithmetic on u = (r + 1/2) / 2^rbits."""
    bits, L = 2, 3
    for log2c in (2, 3):
        c = 1 << log2c
        rng = np.random.default_rng(log2c)
        y = rng.uniform(-1, 1, size=c)
        y[0] = 1.0
        s = np.array([1.0])
        v = (y + 1.0) * (L / 2.0)
        ups = np.zeros(c, dtype=np.int64)
        R = 1 << rbits
        for r in range(R):
            idx = quantize(y, s, log2c, 0, 0, bits, rbits=rbits, r=np.full(c, r))
            assert ((idx == np.floor(v)) | (idx == np.floor(v) + 1) | (idx == L)).all()
            ups += (idx > np.floor(v))
        for j in range(c):
            f = Fraction(float(v[j])) - int(np.floor(v[j]))
            want = sum(1 for r in range(R) if Fraction(2 * r + 1, 2 * R) + f >= 1) if v[j] < L else 0
            assert ups[j] == want
            assert abs(ups[j] / R - float(f)) <= 0.5 / R + 1e-15 or v[j] >= L


def test_rounding_probability_exact_on_the_random_grid():
    """frac(v) a multiple of 2^-RBITS: P(up) equals it exactly."""
    bits, L, log2c = 4, 15, 4
    c = 16
    s = np.array([7.5])
    fr = np.arange(c) / 16.0 + 1 / 256.0
    y = 3 + fr - 7.5
    R = 1 << RBITS
    ups = np.zeros(c)
    for r in range(R):
        ups += quantize(y, s, log2c, 0, 0, bits, r=np.full(c, r)) == 4
    assert (ups / R == fr).all()


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_indices_in_range_and_error_below_one_step(dtype):
    rng = np.random.default_rng(0)
    log2c, bits = 10, 4
    L = 15
    x = (rng.standard_t(3, size=5000) * 1e-3).astype(np.float32)
    y = rht_forward(x, log2c, 9, dtype=dtype)
    s = chunk_absmax(y, log2c)
    idx = quantize(y, s, log2c, 0, 9, bits, dtype=dtype)
    assert idx.min() >= 0 and idx.max() <= L
    step = np.repeat(2 * s.astype(np.float64) / L, 1 << log2c)
    yhat = idx * step - np.repeat(s.astype(np.float64), 1 << log2c)
    assert (np.abs(yhat - y) < step * (1 + 1e-5)).all()
    # the extreme coordinate of each chunk sits on a grid end
    a = np.abs(y).reshape(-1, 1 << log2c)
    am = a.argmax(axis=1)
    ends = idx.reshape(-1, 1 << log2c)[np.arange(len(am)), am]
    assert set(ends.tolist()) <= {0, L}


def test_all_zero_chunk_gives_zero_payload_and_decodes_to_zero():
    log2c, bits = 6, 4
    c = 64
    x = np.zeros(3 * c, dtype=np.float32)
    x[c:2 * c] = np.random.default_rng(0).standard_normal(c)
    for dtype in (np.float64, np.float32):
        out = pipeline([x, x * 0.5], log2c, 4, bits, dtype=dtype)
        assert out["scale"][0] == 0 and out["scale"][2] == 0 and out["scale"][1] > 0
        i0 = out["idx"][0].reshape(3, c)
        assert (i0[0] == 0).all() and (i0[2] == 0).all()
        assert (out["out"][:c] == 0).all() and (out["out"][2 * c:] == 0).all()
        assert np.isfinite(out["out"]).all()


def test_unbiased_over_many_seeds_with_two_point_variance():
    """E[decode(encode(x))] = x and per-coordinate variance of the rotated-domain
    error is step^2 p (1 - p) <= step^2 / 4, p the (RBITS-resolved) round-up
    probability; checked over 10^4 independent rounding streams (workers of one
    seed: same rotation, own Philox stream)."""
    log2c, bits, L = 3, 4, 15
    c = 8
    rng = np.random.default_rng(5)
    x = rng.standard_normal(c).astype(np.float32)
    seed = 12
    y = rht_forward(x, log2c, seed)
    s = chunk_absmax(y, log2c)
    step = 2 * s[0] / L
    v = (y + s[0]) / step
    f = v - np.floor(v)
    N = 10000
    acc = np.zeros(c)
    acc2 = np.zeros(c)
    for w in range(N):
        idx = quantize(y, s, log2c, w, seed, bits)
        yh = idx * step - s[0]
        acc += yh
        acc2 += (yh - y) ** 2
    mean = acc / N
    # exact expectation with RBITS-resolved probability: |p - f| <= 2^-(RBITS+1)
    se = step * np.sqrt(np.maximum(f * (1 - f), 1e-4) / N)
    assert (np.abs(mean - y) <= 4 * se + step * 2.0 ** -(RBITS + 1)).all()
    var = acc2 / N
    assert (var <= step ** 2 / 4 * 1.1).all()
    inner = (f > 0.05) & (f < 0.95)
    assert np.allclose(var[inner], (step ** 2 * f * (1 - f))[inner], rtol=0.15)
    # and through the whole path (W = 1 decodes, averaged): the estimate of x
    xs = np.zeros(c)
    for w in range(2000):
        idx = quantize(y, s, log2c, w, seed, bits)
        xs += decode(idx, s, 1, c, log2c, seed, bits)
    assert np.abs(xs / 2000 - x).max() < 5 * step / 2 / np.sqrt(2000)


# -------------------------------------------------------------------- pack / aggregate
def test_pack_layout_literal_bytes():
    assert pack([1, 2, 3, 4], 4).tolist() == [0x21, 0x43]
    assert pack([1, 2, 3, 0, 3, 3, 0, 1], 2).tolist() == [0b00111001, 0b01001111]
    assert pack([0, 255, 7], 8).tolist() == [0, 255, 7]
    for bits in (2, 4, 8):
        idx = np.random.default_rng(bits).integers(0, 1 << bits, size=64)
        assert (unpack(pack(idx, bits), bits) == idx).all()
        assert pack(idx, bits).size == 64 * bits // 8


def test_sum_width_rule():
    assert sum_dtype(4, 4) == np.uint8          # 60: the paper's baseline q=4, b=8, n=4
    assert sum_dtype(8, 4) == np.uint8          # 120
    assert sum_dtype(8, 2) == np.uint8          # 24
    assert sum_dtype(17, 4) == np.uint8         # 255
    assert sum_dtype(18, 4) == np.uint16        # 270
    assert sum_dtype(8, 8) == np.uint16         # 2040
    assert sum_dtype(257, 8) == np.uint16       # 65535
    with pytest.raises(ValueError):
        sum_dtype(258, 8)


@pytest.mark.parametrize("bits,W", [(2, 8), (4, 4), (4, 17), (8, 8), (8, 3)])
def test_aggregate_is_the_exact_integer_sum(bits, W):
    rng = np.random.default_rng(W)
    L = (1 << bits) - 1
    idx = [rng.integers(0, L + 1, size=256) for _ in range(W)]
    idx[0][:] = L                                # provoke the maximum
    for w in range(W):
        idx[w][5] = L
    S = aggregate([pack(i, bits) for i in idx], bits)
    want = [sum(int(i[g]) for i in idx) for g in range(256)]      # Python integers
    assert S.tolist() == want
    assert S.dtype == sum_dtype(W, bits)
    assert S[5] == W * L and S.max() <= W * L


def test_decode_of_sums_is_mean_of_single_decodes():
    """Ties the all-reduce form (sum integers, decode once) to the parameter-server
    form (decode each worker, average): they are the same linear map."""
    log2c, bits, W = 7, 4, 5
    rng = np.random.default_rng(8)
    n = 3 * 128 - 17
    xs = [(rng.standard_normal(n) * 10 ** rng.uniform(-3, 0)).astype(np.float32) for _ in range(W)]
    out = pipeline(xs, log2c, 31, bits)
    singles = [decode(out["idx"][w], out["scale"], 1, n, log2c, 31, bits) for w in range(W)]
    assert np.allclose(out["out"], np.mean(singles, axis=0), rtol=0, atol=1e-6 * np.abs(out["out"]).max())
    # and the estimate is close to the true mean: the error energy is below the
    # two-point worst case step^2 / (4 W) per (padded) coordinate
    true = np.mean([x.astype(np.float64) for x in xs], axis=0)
    bound = np.sum((2 * out["scale"] / 15) ** 2) * 128 / (4 * W)
    assert np.sum((out["out"] - true) ** 2) < bound


def test_lossless_when_rotated_values_already_sit_on_the_256_grid():
    log2c, bits = 5, 8
    c = 32
    rng = np.random.default_rng(11)
    k = rng.integers(0, 256, size=2 * c)
    k[0], k[1] = 0, 255
    k[c], k[c + 1] = 255, 0
    s = np.array([127.5, 127.5 / 64])
    yg = (k.reshape(2, c) * (2 * s[:, None] / 255) - s[:, None]).reshape(-1)
    idx = quantize(yg, s, log2c, 0, 77, bits)
    assert (idx == k).all()
    out = decode(idx, s, 1, 2 * c, log2c, 77, bits)
    # decode returns the un-rotated vector; rotating it again gives the grid values
    assert np.allclose(rht_forward(out.astype(np.float64), log2c, 77), yg, atol=1e-12 * 127.5)


def test_identical_workers_with_frozen_noise():
    log2c, bits, W = 6, 4, 6
    c = 64
    rng = np.random.default_rng(13)
    x = rng.standard_normal(2 * c).astype(np.float32)
    y = rht_forward(x, log2c, 3)
    s = chunk_absmax(y, log2c)
    r = np.full(2 * c, 127)
    idx = quantize(y, s, log2c, 0, 3, bits, r=r)
    S = aggregate([pack(idx, bits)] * W, bits)
    assert (S == W * idx).all()
    one = decode(idx, s, 1, 2 * c, log2c, 3, bits)
    many = decode(S, s, W, 2 * c, log2c, 3, bits)
    assert np.allclose(one, many, rtol=0, atol=1e-14)
    # u ~ 1/2 is round-to-nearest: error at most half a step (+ the 1/512 offset of u)
    step = np.repeat(2 * s / 15, c)
    assert (np.abs(idx * step - np.repeat(s, c) - y) <= step * (0.5 + 1 / 256)).all()


def test_error_level_matches_two_point_prediction():
    """vNMSE of the W-worker estimate against the closed form
    sum_g step_p^2 f_g (1 - f_g) / W^2 summed over workers / ||mean||^2
    (rotation is orthonormal, so rotated-domain error energy = error energy)."""
    log2c, bits, W = 10, 4, 8
    c, L = 1024, 15
    rng = np.random.default_rng(21)
    n = 8 * c
    xs = [(rng.standard_t(3, size=n) * 1e-3).astype(np.float32) for _ in range(W)]
    out = pipeline(xs, log2c, 6, bits)
    true = np.mean([x.astype(np.float64) for x in xs], axis=0)
    vnmse = np.sum((out["out"] - true) ** 2) / np.sum(true ** 2)
    step = np.repeat(2 * out["scale"] / L, c)
    pred = 0.0
    for w in range(W):
        v = (out["y"][w] + np.repeat(out["scale"], c)) / step
        f = v - np.floor(v)
        pred += np.sum(step ** 2 * f * (1 - f))
    pred = pred / W ** 2 / np.sum(true ** 2)
    assert 0.9 < vnmse / pred < 1.1


def test_scale_is_shared_max_over_workers():
    a = np.array([[1.0, 0.0, 3.0], [2.0, 0.0, 1.0]])
    assert scale_reduce(a).tolist() == [2.0, 0.0, 3.0]
    y = np.array([1.0, -4.0, 2.0, 0.5, 0, 0, 0, -0.25])
    assert chunk_absmax(y, 2).tolist() == [4.0, 0.25]


# ------------------------------------------------------------ fused multiply-add helper
def _rn32(F):
    """Correct rounding of an exact rational to float32 (nearest, ties to even)."""
    c = np.float32(float(F))
    cands = {np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))}
    best = None
    for x in cands:
        d = abs(Fraction(float(x)) - F)
        even = (int(np.float32(x).view(np.uint32)) & 1) == 0
        key = (d, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, x)
    return best[1]


def test_fma32_is_correctly_rounded_against_exact_rationals():
    from oracle.thc import fma32
    rng = np.random.default_rng(12)
    n = 3000
    a = (rng.normal(size=n) * 10.0 ** rng.integers(-6, 6, size=n)).astype(np.float32)
    b = (rng.normal(size=n) * 10.0 ** rng.integers(-6, 6, size=n)).astype(np.float32)
    c = (rng.normal(size=n) * 10.0 ** rng.integers(-6, 6, size=n)).astype(np.float32)
    c[::3] = (-a[::3].astype(np.float64) * b[::3].astype(np.float64)).astype(np.float32)   # heavy cancellation
    got = fma32(a, b, c)
    for i in range(n):
        want = _rn32(Fraction(float(a[i])) * Fraction(float(b[i])) + Fraction(float(c[i])))
        assert got[i] == want, (a[i], b[i], c[i], got[i], want)


def test_fma32_breaks_float64_ties_by_the_discarded_bits():
    """a * b + c lies a hair below (above) the midpoint of two float32 numbers, but the
    float64 sum lands exactly on it: rounding that sum to float32 would go to the even
    neighbour, the fused operation must go down (up)."""
    from oracle.thc import fma32
    a = np.float32(2.0 ** -12 * (1 + 2.0 ** -23))
    b = np.float32(2.0 ** -12 * (1 - 2.0 ** -23))            # a * b = 2^-24 (1 - 2^-46)
    c = np.float32(1 + 2.0 ** -23)
    exact_sum_64 = np.float64(a) * np.float64(b) + np.float64(c)
    assert exact_sum_64 == 1 + 2.0 ** -23 + 2.0 ** -24                           # the midpoint, in float64
    assert np.float32(exact_sum_64) == np.float32(1 + 2.0 ** -22)                # naive: ties to even, up
    assert fma32(a, b, c) == np.float32(1 + 2.0 ** -23)                          # fused: just below -> down
    assert fma32(-a, b, -c) == np.float32(-(1 + 2.0 ** -23))                     # mirrored: e > 0
    assert fma32(a, b, c) == _rn32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


# ------------------------------------------- fp32 evaluation order against the definition
def _quantizer_samples(bits, count, seed):
    """(y, s, r) triples: scales over 2^-120 .. 2^105, y uniform on the range for one half
    of the samples and crowded into the two lowest and two highest grid cells for the other half
    (where a relative error in the multiplier shows most), y = +-s included."""
    rng = np.random.default_rng(1000 * seed + bits)
    L = (1 << bits) - 1
    e = rng.integers(-120, 106, size=count)
    s = (rng.uniform(1.0, 2.0, size=count) * np.exp2(e.astype(np.float64))).astype(np.float32)
    frac = rng.uniform(-1.0, 1.0, size=count)
    edge = rng.uniform(0.0, 4.0 / L, size=count // 2)            # within 2 cells of an end
    frac[: 3 * count // 8] = -1.0 + edge[: 3 * count // 8]       # mostly the low end: there the
    frac[3 * count // 8: count // 2] = 1.0 - edge[3 * count // 8:]   # band is narrowest
    frac[-2000:-1000], frac[-1000:] = 1.0, -1.0
    y = np.clip((s.astype(np.float64) * frac).astype(np.float32), -s, s)
    r = rng.integers(0, 1 << RBITS, size=count)
    return y, s, r


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_fp32_evaluation_orders_against_the_float64_definition(bits):
    """The canonical fp32 order may move an index only where the definition's pre-rounding
    value t lies within 1e-6 * max(1, |t|) of an integer (the band inside which an index is
    allowed to differ).  Measured on 4 x 10^6 triples per grid size (1.2 x 10^7 in all), for
    three evaluation orders written out here in NumPy float32:
      three   ((y + s) * inv) + u, three roundings (add, multiply, add)
      single  fma(y, inv, L/2 + u)
      offset  fma(y + s, inv, u)
    The canonical order (single for L <= 31, offset above) must stay inside the band, and
    `three` must agree with it outside the band; `single` on the 256-point grid does NOT
    stay inside (why the canonical order switches there) - the sample has to show that too,
    otherwise it would not be able to tell the orders apart."""
    from oracle.thc import SINGLE_FMA_MAX_LEVELS, fma32
    L = (1 << bits) - 1
    count = 4_000_000
    y, s, r = _quantizer_samples(bits, count, 7)
    f32 = np.float32
    u = (r.astype(f32) + f32(0.5)) * f32(2.0 ** -RBITS)
    inv = f32(L) / (s + s)
    assert inv.dtype == f32
    floor_idx = lambda t: np.minimum(np.floor(t), f32(L)).astype(np.int64)
    three = floor_idx(((y + s) * inv) + u)
    single = floor_idx(fma32(y, inv, f32(L / 2.0) + u))
    offset = floor_idx(fma32(y + s, inv, u))
    canonical = quantize(y, s, 0, 0, 0, bits, dtype=f32, r=r).astype(np.int64)      # chunks of one
    assert np.array_equal(canonical, single if L <= SINGLE_FMA_MAX_LEVELS else offset)
    y64, s64 = y.astype(np.float64), s.astype(np.float64)
    t64 = y64 * (L / (s64 + s64)) + L / 2.0 + (r + 0.5) / (1 << RBITS)
    definition = np.minimum(np.floor(t64), L).astype(np.int64)
    assert np.array_equal(definition, quantize(y64, s64, 0, 0, 0, bits, dtype=np.float64, r=r))
    outside = np.abs(t64 - np.rint(t64)) > 1e-6 * np.maximum(1.0, np.abs(t64))
    report = {}
    for name, idx in (("three", three), ("single", single), ("offset", offset)):
        moved = idx != definition
        assert (np.abs(idx - definition) <= 1).all()
        report[name] = (int(moved.sum()), int((moved & outside).sum()))
    print(f"bits {bits}: indices moved (in all, outside the band) of {count}: {report}")
    assert report["three"][1] == 0 and report["offset"][1] == 0
    assert ((canonical != definition) & outside).sum() == 0
    assert ((three != canonical) & outside).sum() == 0
    if L <= SINGLE_FMA_MAX_LEVELS:
        assert report["single"][1] == 0
    else:
        assert report["single"][1] > 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_ranges_too_small_for_the_reciprocal_step_are_sent_as_empty(bits, dtype):
    """Reading R7: the rule needs L / (2 s), which binary32 cannot hold for tiny s (255 / 2^-121
    = 2^128.99 overflows; at 2 s = 2^-119 every grid of this library still has a finite
    reciprocal step).  Below MIN_RANGE a chunk is quantized like an all-zero one; at
    MIN_RANGE the ordinary rule applies, end points included, and nothing overflows."""
    from oracle.thc import MIN_RANGE
    L = (1 << bits) - 1
    assert MIN_RANGE == 2.0 ** -119
    with np.errstate(over="ignore"):
        assert np.isinf(np.float32(255.0) / np.float32(2.0 ** -121))
    for levels in (2, 3, 14, 15, 254, 255):
        assert np.isfinite(np.float32(levels) / np.float32(MIN_RANGE))
    c = 16
    rng = np.random.default_rng(bits)
    frac = rng.uniform(-1.0, 1.0, size=c)
    frac[0], frac[1] = 1.0, -1.0
    for two_s, empty in ((2.0 ** -120, True), (np.nextafter(np.float32(2.0 ** -119), np.float32(0)), True),
                         (2.0 ** -119, False), (2.0 ** -100, False)):
        s = dtype(two_s) / dtype(2)
        y = (frac * float(s)).astype(dtype)
        with np.errstate(all="raise"):
            idx, t = quantize(y, [s], 4, 0, 9, bits, dtype=dtype, return_t=True)
        if empty:
            assert (idx == 0).all()
        else:
            assert np.isfinite(t).all()
            assert idx[0] == L and idx[1] == 0 and idx.max() <= L
            step = float(two_s) / L
            back = idx.astype(np.float64) * step - float(s)
            assert (np.abs(back - y.astype(np.float64)) <= step * (1 + 1e-6)).all()
    # through the whole path: the chunk keeps its (tiny) scale, is sent as zeros, and the
    # estimate of the mean is off by at most the range itself per rotated coordinate
    xs = [(rng.uniform(-1.0, 1.0, size=32) * 2.0 ** -124).astype(np.float32) for _ in range(3)]
    res = pipeline(xs, 4, 7, bits, dtype=dtype)
    assert (res["scale"] > 0).all() and (2 * res["scale"] < MIN_RANGE).all()
    assert all(int(p.max()) == 0 for p in res["payloads"])
    mean = np.mean(np.stack(xs).astype(np.float64), axis=0)
    assert np.abs(res["out"] - mean).max() <= 4 * 2.0 ** -119      # 1/sqrt(16) * 16 terms of at most 2^-119


@pytest.mark.parametrize("bits", [2, 4])
def test_pipeline_with_a_partial_last_payload_byte(bits):
    """Chunks of 2 coordinates, an odd number of them: the payload's last byte is only partly
    used (10 coordinates x 2 bits = 2.5 bytes); the unused bits are no coordinates, the sums
    have one entry per padded coordinate, and the estimate is the mean of the workers' own."""
    W, n, l = 3, 9, 1
    rng = np.random.default_rng(bits)
    xs = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    res = pipeline(xs, l, 3, bits, dtype=np.float64)
    assert res["sums"].size == 10 and len(res["scale"]) == 5
    assert all(p.size == (10 * bits + 7) // 8 for p in res["payloads"])
    singles = [decode(aggregate([p], bits, count=10), res["scale"], 1, n, l, 3, bits) for p in res["payloads"]]
    assert np.allclose(res["out"], np.mean(singles, axis=0), rtol=0, atol=1e-12)
