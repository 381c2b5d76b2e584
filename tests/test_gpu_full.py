"""Full rotation (one chunk = the whole padded gradient) on the GPU against the oracle run
with chunk_log2 = log2_size: rotated values, payloads, sums and output bit-identical to
the fp32 canonical order; output within 1e-5 relative L2 of the float64 definition."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from synth import to_numpy_bits

from gpu_util import DEV, sums_to_numpy

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


@pytest.mark.parametrize("l,n,dtype", [
    (15, 1 << 15, torch.float32), (15, 20_001, torch.bfloat16), (16, 40_000, torch.float32),
    (17, 100_003, torch.bfloat16), (20, 777_777, torch.float32), (23, (1 << 23) - 5, torch.bfloat16),
    (24, 9_000_001, torch.float32), (18, 1, torch.float32), (19, (1 << 14) + 1, torch.bfloat16),
])
def test_full_rotation_forward_and_inverse(l, n, dtype):
    print(f"full rotation l={l} n={n} dtype={dtype}", flush=True)
    assert thc.thc_full_log2(n) <= l
    x = _rand(n, dtype, 11 * l)
    size = 1 << l
    y = torch.full((size,), float("nan"), device=DEV)
    thc.rht_forward_full(x, l, 7, y)
    torch.cuda.synchronize()
    hx = to_numpy_bits(x)
    bf16 = dtype == torch.bfloat16
    ref = O.rht_forward(hx, l, 7, dtype=np.float32, bf16=bf16)
    got = y.cpu().numpy()
    assert (got == ref).all(), f"{int((got != ref).sum())} rotated values differ"
    y64 = O.rht_forward(hx, l, 7, dtype=np.float64, bf16=bf16)
    assert np.linalg.norm(got - y64) <= 1e-5 * np.linalg.norm(y64)

    back = torch.full((n,), float("nan"), device=DEV)
    thc.rht_inverse_full(y, n, l, 7, back)     # y is scratch from here on
    torch.cuda.synchronize()
    ref_back = O.rht_inverse(ref, n, l, 7, dtype=np.float32)
    assert (back.cpu().numpy() == ref_back).all()
    xf = x.float().cpu().numpy().astype(np.float64)
    assert np.linalg.norm(back.cpu().numpy() - xf) <= 1e-5 * max(np.linalg.norm(xf), 1e-30)


@pytest.mark.parametrize("l,n,W,bits,dtype", [
    (15, 30_000, 3, 4, torch.float32), (18, 200_001, 4, 4, torch.bfloat16),
    (21, 1_500_000, 2, 8, torch.bfloat16), (16, 1 << 16, 18, 4, torch.float32), (17, 99_999, 3, 2, torch.float32),
    (20, 5_000, 2, 4, torch.float32), (22, 70_001, 3, 2, torch.bfloat16),   # mostly implied padding
])
def test_full_rotation_pipeline_matches_oracle(l, n, W, bits, dtype):
    _full_pipeline(l, n, W, bits, dtype)


def _full_pipeline(l, n, W, bits, dtype, magnitude=1.0):
    print(f"full pipeline l={l} n={n} W={W} bits={bits} dtype={dtype} magnitude={magnitude}", flush=True)
    size = 1 << l
    xs = [(_rand(n, torch.float32, 100 * l + w, scale=10.0 ** (-1 - (w % 3))) * magnitude).to(dtype) for w in range(W)]
    absmax = torch.empty(W, device=DEV)
    scale = torch.empty(1, device=DEV)
    ys = [torch.full((size,), float("nan"), device=DEV) for _ in range(W)]   # the padding is not pre-zeroed
    nb = size * bits // 8
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sb = thc.thc_sum_bytes(W, bits)
    sums = torch.empty(size, dtype=torch.uint8 if sb == 1 else torch.int16, device=DEV)
    out = torch.empty(n, device=DEV)
    for w in range(W):
        if w % 2 == 0:                     # both forms: rotation and range in one call, or in two
            absmax[w] = float("nan")
            thc.rht_forward_full_absmax(xs[w], l, 9, ys[w], absmax[w:w + 1])
        else:
            thc.rht_forward_full(xs[w], l, 9, ys[w])
            thc.thc_full_absmax(ys[w], l, absmax[w:w + 1])
    thc.thc_scale_reduce(absmax, W, 1, scale)
    for w in range(W):
        thc.thc_full_encode(ys[w], l, 9, w, bits, scale, payloads[w])
    # the deferred form: the last pass first evaluated for the range only, then again for the payload
    work = torch.full((size,), float("nan"), device=DEV)
    for w in range(W):
        range_only = torch.full((1,), float("nan"), device=DEV)
        thc.rht_forward_full_deferred(xs[w], l, 9, work, range_only)
        payload = torch.full((nb,), 0x55, dtype=torch.uint8, device=DEV)
        thc.thc_full_encode_deferred(work, n, l, 9, w, bits, scale, payload)
        assert float(range_only[0]) == float(absmax[w]), f"range of worker {w}"
        assert torch.equal(payload, payloads[w]), f"deferred payload {w}"
    del work
    thc.thc_aggregate(payloads, size, 14, bits, sums)
    yhat = ys[0]
    thc.thc_full_decode(sums, scale, W, l, bits, yhat)
    thc.rht_inverse_full(yhat, n, l, 9, out)
    out_one_call = torch.full((n,), float("nan"), device=DEV)      # the same two steps as one call
    thc.thc_full_decode_inverse(sums, scale, W, n, l, 9, bits, ys[-1].fill_(float("nan")), out_one_call)
    torch.cuda.synchronize()
    assert torch.equal(out, out_one_call)

    bf16 = dtype == torch.bfloat16
    ref = O.pipeline([to_numpy_bits(x) for x in xs], l, 9, bits, dtype=np.float32, bf16=bf16)
    assert scale.cpu().numpy()[0] == ref["scale"][0]
    for w in range(W):
        assert (payloads[w].cpu().numpy() == ref["payloads"][w]).all(), f"payload {w}"
    assert (sums_to_numpy(sums) == ref["sums"]).all()
    assert (out.cpu().numpy() == ref["out"]).all()
    d64 = O.decode(ref["sums"], ref["scale"].astype(np.float64), W, n, l, 9, bits)
    assert np.linalg.norm(out.cpu().numpy() - d64) <= 1e-5 * np.linalg.norm(d64)
    return float(scale[0]), payloads


@pytest.mark.parametrize("l,n,W,bits,dtype", [(15, 30_000, 3, 4, torch.float32), (15, 30_000, 3, 8, torch.bfloat16),
                                               (16, 40_260, 8, 4, torch.float32), (19, 355_054, 18, 8, torch.float32)])
def test_full_rotation_of_a_vanishingly_small_gradient(l, n, W, bits, dtype):
    """A whole gradient whose scale is below 2^-120 (L / (2 s) is not finite in fp32): sent as
    zeros, as the oracle does.  The rotated values are subnormal, so the normalisation must be
    the single multiplication after the last stage that the oracle performs: a factor 2^-7
    taken after the first 14 stages would round there (the last two shapes caught that)."""
    s, payloads = _full_pipeline(l, n, W, bits, dtype, magnitude=2.0 ** -128)
    assert 0 < s < 2.0 ** -121
    assert all(int(p.max()) == 0 for p in payloads)


def test_full_rotation_randomized_shapes_and_magnitudes():
    """Fixed-seed random cases: sizes from a handful of coordinates to a full power of two
    (so from almost all padding to none), 1 to 18 workers, every payload width, magnitudes
    from below the smallest range the quantizer accepts to 2^80; both forms of every step."""
    import random
    rnd = random.Random(11)
    for _ in range(30):
        l = rnd.choice([15, 15, 16, 17, 18, 19, 20, 21, 23, 24])
        n = rnd.choice([rnd.randint((1 << (l - 1)) + 1, 1 << l), rnd.randint(1, 1 << l), min(1 << l, rnd.randint(1, 70000))])
        W = rnd.choice([1, 2, 3, 8, 18]) if l < 21 else rnd.choice([1, 2, 3])
        bits = rnd.choice([2, 4, 8])
        dtype = rnd.choice([torch.float32, torch.bfloat16])
        magnitude = rnd.choice([2.0 ** -128, 2.0 ** -117, 1e-20, 1.0, 1.0, 2.0 ** 80])
        with np.errstate(all="ignore"):
            _full_pipeline(l, n, W, bits, dtype, magnitude=magnitude)


def test_full_rotation_of_an_empty_gradient():
    """n = 0: the rotated vector is all zeros, its range 0, its payload all index 0."""
    l = 16
    x = torch.empty(0, device=DEV)
    y = torch.full((1 << l,), float("nan"), device=DEV)
    absmax = torch.full((2,), float("nan"), device=DEV)
    thc.rht_forward_full_absmax(x, l, 3, y, absmax[0:1])
    assert float(y.abs().max()) == 0.0 and float(absmax[0]) == 0.0
    work = torch.full((1 << l,), float("nan"), device=DEV)
    thc.rht_forward_full_deferred(x, l, 3, work, absmax[1:2])
    assert float(absmax[1]) == 0.0
    payload = torch.full(((1 << l) // 2,), 0xAA, dtype=torch.uint8, device=DEV)
    thc.thc_full_encode_deferred(work, 0, l, 3, 0, 4, absmax[1:2], payload)
    assert int(payload.max()) == 0


def test_full_rotation_argument_checks():
    y = torch.empty(1 << 15, device=DEV)
    x = torch.empty(100, device=DEV)
    with pytest.raises(thc.ThcError):
        thc.rht_forward_full(x, 14, 0, y)          # log2_size below 15
    with pytest.raises(thc.ThcError):
        thc.rht_forward_full(torch.empty((1 << 15) + 4, device=DEV), 15, 0, y)   # n > 2^l
    with pytest.raises(thc.ThcError):
        thc.rht_forward_full(x[1:], 15, 0, y)      # x not 16-byte aligned
    sums = torch.empty(1 << 15, dtype=torch.uint8, device=DEV)
    scale = torch.ones(1, device=DEV)
    with pytest.raises(thc.ThcError):
        thc.thc_full_decode_inverse(sums, scale, 3, 100, 15, 0, 4, y[1:], x)      # scratch not 16-byte aligned
    with pytest.raises(thc.ThcError):
        thc.thc_full_decode_inverse(sums, scale, 3, 100, 15, 0, 5, y, x)          # bits
    with pytest.raises(thc.ThcError):
        thc.thc_full_decode_inverse(sums, scale, 300, 100, 15, 0, 8, y, x)        # sums of 300 workers do not fit 16 bits
    with pytest.raises(thc.ThcError):
        thc.thc_full_decode_inverse(sums, scale, 3, (1 << 15) + 1, 15, 0, 4, y, x)   # n > 2^l


def test_full_rotation_over_2_to_33_coordinates():
    """One rotation over 2^33 coordinates (n just above 2^32): element indices need 33 bits.
    The input is zero except for a few exactly representable entries, so every output value
    has the closed form  y_i = N^(-1/2) * sum_j D_kj x_kj (-1)^popcount(i & kj)  (a few terms,
    exact before the final scaling), checked at positions on both sides of 2^32; the
    inverse must then give the input back."""
    l = 33
    n = (1 << 32) + 12_345
    assert thc.thc_full_log2(n) == l
    ks = [0, 5, (1 << 14) + 3, (1 << 31) + 7, (1 << 32) + 11, n - 1]
    vs = [1.0, -2.0, 0.5, 4.0, 1.0, -1.0]
    x = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    for k, v in zip(ks, vs):
        x[k] = v
    y = torch.empty(1 << l, device=DEV)
    print(f"full rotation l={l} n={n}", flush=True)
    thc.rht_forward_full(x, l, 9, y)
    torch.cuda.synchronize()
    signed = [(-v if O.sign_bits(k, 1, 9)[0] else v) for k, v in zip(ks, vs)]
    rng = np.random.default_rng(0)
    probe = [0, 1, (1 << 14) - 1, 1 << 14, (1 << 32) - 1, 1 << 32, (1 << 32) + 11, (1 << 33) - 1]
    probe += [int(i) for i in rng.integers(0, 1 << 33, size=200)]
    got = y[torch.tensor(probe, device=DEV)].cpu().numpy().astype(np.float64)
    want = np.array([sum(s * (-1) ** bin(i & k).count("1") for s, k in zip(signed, ks)) for i in probe],
                    dtype=np.float64) * 2.0 ** -16.5
    assert np.abs(got - want).max() <= 1e-6 * np.abs(want).max()
    # energy: the rotation is orthonormal (sum over all 2^33 outputs, in float64 on the device)
    step = 1 << 28
    energy = sum(float((y[a:a + step].double() ** 2).sum()) for a in range(0, 1 << l, step))
    assert abs(energy - sum(v * v for v in vs)) <= 1e-5 * sum(v * v for v in vs)
    scale = torch.empty(1, device=DEV)
    thc.thc_full_absmax(y, l, scale)
    stored = torch.empty((1 << l) // 2, dtype=torch.uint8, device=DEV)
    thc.thc_full_encode(y, l, 9, 3, 4, scale, stored)
    back = torch.full((n,), float("nan"), device=DEV)
    thc.rht_inverse_full(y, n, l, 9, back)
    torch.cuda.synchronize()
    err2 = sum(float(((back[a:a + step] - x[a:a + step].float()).double() ** 2).sum()) for a in range(0, n, step))
    assert err2 ** 0.5 <= 1e-5 * sum(v * v for v in vs) ** 0.5
    del back
    # the deferred form at this size (y is scratch by now): same range, same payload bytes
    range_only = torch.empty(1, device=DEV)
    thc.rht_forward_full_deferred(x, l, 9, y, range_only)
    deferred = torch.empty((1 << l) // 2, dtype=torch.uint8, device=DEV)
    thc.thc_full_encode_deferred(y, n, l, 9, 3, 4, scale, deferred)
    torch.cuda.synchronize()
    assert float(range_only[0]) == float(scale[0]) > 0
    assert all(torch.equal(stored[a:a + step], deferred[a:a + step]) for a in range(0, (1 << l) // 2, step))
