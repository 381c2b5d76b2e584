"""Pins for the oracle of the min/max-range variant (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import thc as T
from oracle.thc_minmax import (chunk_minmax, decode_minmax, maybe_rotate, pipeline_minmax,
                               quantize_minmax, range_reduce, to_bf16_bits)


def test_chunk_minmax_and_range_reduce_literal():
    y = np.array([1.0, -3.0, 2.0, 0.5, 7.0, 7.5, 6.0, 9.0])
    assert chunk_minmax(y, 2).tolist() == [[-3.0, 2.0], [6.0, 9.0]]
    allr = np.array([[[-3.0, 2.0], [6.0, 9.0]], [[-1.0, 5.0], [4.0, 8.0]]])
    assert range_reduce(allr).tolist() == [[-3.0, 5.0], [4.0, 9.0]]


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_symmetric_range_reproduces_the_symmetric_quantizer(bits, dtype):
    """With lo = -s and hi = +s the two grids are the same grid.  The min/max form is
    t = fma(fl(y - lo), inv, u).  On the 256-point grid the symmetric quantizer takes the
    same offset form, so the indices are identical.  On the smaller grids it evaluates
    t' = fma(y, inv, L/2 + u), and the two values differ only by rounding, eps = one
    rounding error of the arithmetic (2^-24 in fp32, 2^-53 in float64):
      t'  carries  (L/2) eps  (inv's rounding error times |y inv| <= L/2) + |t| eps  (its own rounding),
      t   carries  |t| eps (y - lo) + |t| eps (inv) + |t| eps (its own rounding),
    so |t - t'| <= (L/2 + 4 max(1, |t|)) eps, and an index can differ only where t' lies
    that close to an integer."""
    log2c, seed = 8, 3
    L = (1 << bits) - 1
    eps = 2.0 ** -24 if dtype == np.float32 else 2.0 ** -53
    rng = np.random.default_rng(bits)
    y = rng.normal(size=40 << log2c).astype(dtype)
    s = T.chunk_absmax(y, log2c).astype(dtype)
    sym, t = T.quantize(y, s, log2c, 2, seed, bits, dtype=dtype, return_t=True)
    mm = quantize_minmax(y, np.stack([-s, s], axis=1), log2c, 2, seed, bits, dtype=dtype)
    differ = np.flatnonzero(sym != mm)
    if L > T.SINGLE_FMA_MAX_LEVELS and dtype == np.float32:
        assert differ.size == 0
    assert differ.size <= 3
    t = t.astype(np.float64)
    bound = (L / 2.0 + 4.0 * np.maximum(1.0, np.abs(t[differ]))) * eps
    assert (np.abs(t[differ] - np.rint(t[differ])) <= bound).all()
    assert (np.abs(sym[differ].astype(int) - mm[differ].astype(int)) == 1).all()
    sums = T.aggregate([T.pack(sym, bits)], bits)
    a = T.decode(sums, s, 1, y.size, log2c, seed, bits, dtype=np.float64)
    b = decode_minmax(sums, np.stack([-s, s], axis=1), 1, y.size, log2c, seed, bits, True, dtype=np.float64)
    assert np.allclose(a, b, rtol=0, atol=1e-12)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_end_points_and_grid_points_for_every_random_value(bits):
    L = (1 << bits) - 1
    log2c, c = 6, 64
    lo, hi = -0.25, 1.75
    rng = np.array([[lo, hi]])
    grid = lo + (hi - lo) * (np.arange(c) % (L + 1)) / L
    for r in range(256):
        rr = np.full(c, r)
        assert (quantize_minmax(np.full(c, lo), rng, log2c, 0, 0, bits, r=rr) == 0).all()
        assert (quantize_minmax(np.full(c, hi), rng, log2c, 0, 0, bits, r=rr) == L).all()
    idx = quantize_minmax(grid, rng, log2c, 0, 0, bits, r=np.full(c, 0))
    assert (idx == np.arange(c) % (L + 1)).all()


def test_shift_invariance_of_indices():
    """Moving the data and its range by the same exactly representable amount leaves the
    indices unchanged (the symmetric grid has no such property: that is the point of
    carrying lo and hi)."""
    log2c, bits = 7, 4
    rng = np.random.default_rng(1)
    y = rng.integers(-1000, 1000, size=3 << log2c).astype(np.float64) / 1024.0
    r = chunk_minmax(y, log2c)
    base = quantize_minmax(y, r, log2c, 1, 5, bits)
    shifted = quantize_minmax(y + 4.0, r + 4.0, log2c, 1, 5, bits)
    assert (base == shifted).all()


def test_degenerate_range_decodes_to_the_constant():
    log2c, bits, W = 5, 4, 3
    xs = [np.full(40, 0.375, dtype=np.float32) for _ in range(W)]
    res = pipeline_minmax(xs, log2c, 0, bits, rotate=False)
    assert (res["range"][0] == [0.375, 0.375]).all()          # full chunk: constant
    assert (res["idx"][0][:32] == 0).all()
    assert (res["out"][:32] == 0.375).all()
    assert res["range"][1].tolist() == [0.0, 0.375]            # ragged chunk: zero padding widens it


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_range_too_narrow_for_the_reciprocal_step_is_sent_as_constant(dtype):
    """M2: below MIN_RANGE = 2^-119 the range is treated like an empty one (L / width need not
    be finite in binary32): indices 0, decoded to lo, at most the width away; at MIN_RANGE
    the ordinary rule applies and the end points get 0 and L."""
    from oracle.thc_minmax import quantize_minmax
    bits, L, c = 8, 255, 8
    lo = dtype(3.0) * dtype(2.0 ** -118)
    for width, empty in ((2.0 ** -120, True), (2.0 ** -119, False)):
        hi = lo + dtype(width)
        assert hi - lo == dtype(width)
        y = np.linspace(float(lo), float(hi), c).astype(dtype)
        y[0], y[-1] = lo, hi
        with np.errstate(all="raise"):
            idx = quantize_minmax(y, [[lo, hi]], 3, 0, 4, bits, dtype=dtype)
        if empty:
            assert (idx == 0).all()
            out = decode_minmax(idx.astype(np.int64), [[lo, hi]], 1, c, 3, 4, bits, False, dtype=dtype)
            assert (np.abs(out.astype(np.float64) - y.astype(np.float64)) <= width).all()
        else:
            assert idx[0] == 0 and idx[-1] == L


def test_single_worker_error_below_one_step_with_and_without_rotation():
    log2c, bits = 8, 4
    rng = np.random.default_rng(2)
    x = (rng.normal(size=1000) + 3.0).astype(np.float32)        # far from zero-mean
    for rotate in (True, False):
        res = pipeline_minmax([x], log2c, 7, bits, rotate=rotate)
        y = res["y"][0].reshape(-1, 1 << log2c)
        step = ((res["range"][:, 1] - res["range"][:, 0]) / 15).reshape(-1, 1)
        yhat = res["sums"].astype(float).reshape(y.shape) * step + res["range"][:, 0:1]
        assert (np.abs(yhat - y) <= step * (1 + 1e-12)).all()
    # no rotation: the estimate lives in the input domain directly
    res = pipeline_minmax([x], log2c, 7, bits, rotate=False)
    assert np.abs(res["out"] - x).max() <= ((res["range"][:, 1] - res["range"][:, 0]) / 15).max() * (1 + 1e-6)


def test_no_rotation_means_identity_padding_only():
    x = np.arange(10, dtype=np.float32)
    y = maybe_rotate(x, 3, 99, rotate=False)
    assert y.tolist() == list(range(10)) + [0.0] * 6
    xb = (np.array([1.5, -2.0], dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert maybe_rotate(xb, 1, 0, rotate=False, bf16=True).tolist() == [1.5, -2.0]


def test_minmax_beats_symmetric_on_shifted_data():
    """A chunk whose values sit far from zero wastes most of a symmetric grid; the
    min/max grid does not (closed form: error scales with the width of the grid)."""
    log2c, bits, W = 8, 4, 4
    rng = np.random.default_rng(3)
    xs = [(rng.normal(size=1 << 12) * 0.1 + 5.0).astype(np.float32) for _ in range(W)]
    mean = np.mean(xs, axis=0)
    mm = pipeline_minmax(xs, log2c, 1, bits, rotate=False)
    ys = [maybe_rotate(x, log2c, 1, False) for x in xs]
    s = T.scale_reduce(np.stack([T.chunk_absmax(y, log2c) for y in ys]))
    sym_idx = [T.quantize(y, s, log2c, w, 1, bits) for w, y in enumerate(ys)]
    sums = T.aggregate([T.pack(i, bits) for i in sym_idx], bits)
    step = (2 * s / 15).reshape(-1, 1)
    sym = (sums.astype(float).reshape(-1, 1 << log2c) * step / W - s.reshape(-1, 1)).reshape(-1)
    err_mm = np.linalg.norm(mm["out"] - mean)
    err_sym = np.linalg.norm(sym - mean)
    assert err_mm < 0.2 * err_sym


def test_bf16_rounding_matches_the_library_conversion():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.normal(size=100_000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, size=100_000),
                        # exact ties and their neighbours
                        (np.arange(0x3F800000, 0x3F800000 + (1 << 18), 1 << 15, dtype=np.uint32)).view(np.float32),
                        np.array([0.0, -0.0, 1.0, -1.0, 65504.0, 1e-40, -1e-40], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (to_bf16_bits(x) == want).all()


def test_fp32_mode_agrees_with_the_definition():
    rng = np.random.default_rng(6)
    xs = [(rng.standard_t(3, size=3000) * 1e-3 + 2e-3).astype(np.float32) for _ in range(4)]
    for rotate in (True, False):
        r64 = pipeline_minmax(xs, 9, 2, 4, rotate=rotate, dtype=np.float64)
        r32 = pipeline_minmax(xs, 9, 2, 4, rotate=rotate, dtype=np.float32)
        mism = sum(int((a != b).sum()) for a, b in zip(r64["idx"], r32["idx"]))
        assert mism <= 2
