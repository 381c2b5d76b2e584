"""CPU oracle of the paper-literal range variant: the grid spans the chunk's minimum to
its maximum, split evenly (the range as the THC background paragraph and the "Partial
rotation" paragraph word it), optionally without any rotation (the "No Rotation" column
of the THC throughput table), with an optional bf16 output.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Readings (the paper fixes only the idea of a min-max range):
  M1  One range per chunk, shared by all workers so that integer sums stay decodable:
      lo_p = min over workers of the chunk's smallest rotated value, hi_p = max over
      workers of its largest.  The header is the pair (lo_p, hi_p).
  M2  Grid: 2^b points, index 0 at lo_p, index L at hi_p; hi_p == lo_p gives inv = 0,
      all indices 0, and decodes to exactly lo_p.  So does a range narrower than
      MIN_RANGE = 2^-119, for which L / (hi - lo) need not be finite in binary32 (reading
      R7 of the symmetric path); it decodes to lo_p, at most its own width away.
          inv = L / (hi - lo);  t = (y - lo) * inv + u;  idx = min(floor(t), L)
      (u as in the symmetric path, same random stream; in the fp32 mode the subtraction
      is one operation and the multiply-add one fused operation).
  M3  Decode: step = (hi - lo) / L;  yhat = S * (step / W) + lo;  then the inverse
      rotation (or nothing when the rotation is off).
  M4  Without rotation the "rotated values" are the (zero-padded) gradient itself: no
      sign diagonal, no butterflies, no normalisation.
  M5  bf16 output: the fp32 result rounded to nearest, ties to even.
"""

import numpy as np

from . import thc as T


def maybe_rotate(x, chunk_log2, seed, rotate, dtype=np.float64, bf16=False, g0=0):
    """M4: rotation on -> the chunked RHT; off -> the widened, zero-padded input."""
    if rotate:
        return T.rht_forward(x, chunk_log2, seed, dtype=dtype, bf16=bf16, g0=g0)
    c = 1 << chunk_log2
    P = T.num_chunks(len(x), chunk_log2)
    a = np.zeros(P * c, dtype=dtype)
    a[:len(x)] = T._widen(x, bf16, dtype)
    return a


def chunk_minmax(y, chunk_log2):
    """(P, 2) array of (min, max) per chunk."""
    c = 1 << chunk_log2
    v = y.reshape(-1, c)
    return np.stack([v.min(axis=1), v.max(axis=1)], axis=1)


def range_reduce(ranges_all):
    """M1: ranges_all (W, P, 2) -> (P, 2): min of the minima, max of the maxima."""
    r = np.asarray(ranges_all)
    return np.stack([r[:, :, 0].min(axis=0), r[:, :, 1].max(axis=0)], axis=1)


def quantize_minmax(y, rng, chunk_log2, worker, seed, bits, dtype=np.float64, g0=0, r=None):
    """M2."""
    c = 1 << chunk_log2
    L = (1 << bits) - 1
    y = np.asarray(y, dtype=dtype).reshape(-1, c)
    rng = np.asarray(rng, dtype=dtype).reshape(-1, 2)
    lo, hi = rng[:, 0:1], rng[:, 1:2]
    width = hi - lo
    inv = np.zeros_like(width)
    nz = width >= dtype(T.MIN_RANGE)             # a constant chunk, or one too narrow for L / width
    inv[nz] = dtype(L) / width[nz]
    if r is None:
        r = T.rounding_fields(g0, y.size, worker, seed)
    r = np.asarray(r).reshape(y.shape)
    u = (r.astype(dtype) + dtype(0.5)) * dtype(2.0 ** -T.RBITS)
    d = y - lo                                   # rounded on its own in the fp32 mode
    t = T.fma32(d, inv, u) if dtype == np.float32 else d * inv + u
    return np.minimum(np.floor(t), dtype(L)).astype(np.uint16).reshape(-1)


def to_bf16_bits(x):
    """M5: fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    return (rounded >> np.uint64(16)).astype(np.uint16)


def decode_minmax(sums, rng, W, n, chunk_log2, seed, bits, rotate, dtype=np.float64, g0=0, out_bf16=False):
    """M3 (+ M5)."""
    c = 1 << chunk_log2
    L = (1 << bits) - 1
    rng = np.asarray(rng, dtype=dtype).reshape(-1, 2)
    lo, hi = rng[:, 0:1], rng[:, 1:2]
    step = (hi - lo) / dtype(L)
    q = step / dtype(W)
    S = np.asarray(sums).reshape(-1, c).astype(dtype)
    yhat = (S * q + lo).reshape(-1)
    out = T.rht_inverse(yhat, n, chunk_log2, seed, dtype=dtype, g0=g0) if rotate else yhat[:n]
    if out_bf16:
        return to_bf16_bits(out.astype(np.float32))
    return out


def pipeline_minmax(xs, chunk_log2, seed, bits, rotate=True, dtype=np.float64, bf16=False, g0=0,
                    out_bf16=False):
    W, n = len(xs), len(xs[0])
    ys = [maybe_rotate(x, chunk_log2, seed, rotate, dtype=dtype, bf16=bf16, g0=g0) for x in xs]
    ranges_all = np.stack([chunk_minmax(y, chunk_log2) for y in ys])
    rng = range_reduce(ranges_all)
    idx = [quantize_minmax(y, rng, chunk_log2, w, seed, bits, dtype=dtype, g0=g0) for w, y in enumerate(ys)]
    payloads = [T.pack(i, bits) for i in idx]
    sums = T.aggregate(payloads, bits, count=idx[0].size)
    out = decode_minmax(sums, rng, W, n, chunk_log2, seed, bits, rotate, dtype=dtype, g0=g0, out_bf16=out_bf16)
    return dict(y=ys, ranges_all=ranges_all, range=rng, idx=idx, payloads=payloads, sums=sums, out=out)
