"""CPU oracle of the saturation-based aggregation variant ("Saturation-based
aggregation" paragraph of the paper's proposed improvements to THC).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

What the paper fixes: partially aggregated values are combined with

    Sat(x, y) = min(2^(b-1) - 1, max(-2^(b-1) + 1, x + y))

on top of the rotated and normalised gradients, with b = q bits, so an
intermediate hop of an all-reduce never needs more than the q bits a worker
sends.  What it leaves open, and the reading taken here (and, independently,
by the GPU library):

  S1  Grid.  Sat's range is the signed symmetric set {-M, ..., M},
      M = 2^(b-1) - 1, i.e. 2^b - 1 levels.  A worker's coordinate is rounded
      onto 2M + 1 evenly spaced points of [-s_p, +s_p]: idx in [0, 2M] with the
      same stochastic rounding rule as the exact-sum path (L replaced by 2M; an all-zero
      chunk lands on the centre index M by the rule itself),
      and z = idx - M is the signed value.  y = 0 sits exactly on a grid point.
  S2  Payload.  idx is stored in b bits (offset binary), packed as in the
      exact-sum path; the all-ones code 2^b - 1 never occurs.
  S3  Order.  Sat is not associative, so the order matters: the aggregate is
      a_0 = z_0, a_w = Sat(a_(w-1), z_w) for w = 1 .. W-1, the order in which a
      ring reduction that starts at worker 0 visits a block.  The result is
      stored offset-binary in b bits: A = a_(W-1) + M.
  S4  Decode.  a estimates the SUM of the workers' signed grid values; the mean
      gradient estimate is yhat = a * (step / W), step = (s_p + s_p) / (2M),
      followed by the inverse rotation.
  S5  "Overflow" of a coordinate = at least one of its W - 1 Sat steps clipped.
"""

import numpy as np

from . import thc as T


def sat_max(bits):
    """M = 2^(b-1) - 1, the largest magnitude Sat lets through (b = q)."""
    return (1 << (bits - 1)) - 1


def sat(x, y, bits):
    """The paper's operator, written out: min(M, max(-M, x + y))."""
    M = sat_max(bits)
    return np.minimum(M, np.maximum(-M, np.asarray(x, dtype=np.int64) + np.asarray(y, dtype=np.int64)))


def sat_quantize(y, scale, chunk_log2, worker, seed, bits, dtype=np.float64, g0=0, r=None):
    """Reading S1: stochastic rounding onto the 2M+1-point grid of [-s_p, s_p].

        inv = 2M / (s_p + s_p)
        t   = y * inv + M + u,  u = (r + 0.5) / 2^RBITS   (fp32 evaluation order and random
                                                           stream of the exact-sum path)
        idx = min(floor(t), 2M);  2 s_p < MIN_RANGE (in particular s_p = 0) -> idx = M
                                  (the grid's centre: z = 0)
    """
    c = 1 << chunk_log2
    L = 2 * sat_max(bits)
    y = np.asarray(y, dtype=dtype).reshape(-1, c)
    s = np.asarray(scale, dtype=dtype).reshape(-1, 1)
    two_s = s + s
    inv = np.zeros_like(two_s)
    nz = two_s >= dtype(T.MIN_RANGE)
    inv[nz] = dtype(L) / two_s[nz]
    if r is None:
        r = T.rounding_fields(g0, y.size, worker, seed)
    r = np.asarray(r).reshape(y.shape)
    u = (r.astype(dtype) + dtype(0.5)) * dtype(2.0 ** -T.RBITS)
    t = T.grid_position_plus_noise(y, s, inv, L, u, dtype)
    idx = np.minimum(np.floor(t), dtype(L)).astype(np.uint16)
    idx[np.broadcast_to(~nz, idx.shape)] = L // 2          # all-zero chunk: the centre, z = 0
    return idx.reshape(-1)


def sat_aggregate(payloads, bits, count=None):
    """Readings S2, S3, S5.  Returns (A, clipped): the offset-binary aggregate
    A = a + M per coordinate (uint16 array of values in [0, 2M]) and a boolean
    array, True where any Sat step clipped."""
    M = sat_max(bits)
    z = [T.unpack(p, bits).astype(np.int64) - M for p in payloads]
    a = z[0].copy()
    clipped = np.zeros(a.shape, dtype=bool)
    for zw in z[1:]:
        raw = a + zw
        a = sat(a, zw, bits)
        clipped |= raw != a
    if count is not None:
        a, clipped = a[:count], clipped[:count]
    assert (np.abs(a) <= M).all()
    return (a + M).astype(np.uint16), clipped


def sat_decode(A, scale, W, n, chunk_log2, seed, bits, dtype=np.float64, g0=0):
    """Reading S4.

        step = (s_p + s_p) / (2M)
        yhat = (A - M) * (step / W)
        xhat = D (1/sqrt(c)) H_c yhat,  first n coordinates
    """
    c = 1 << chunk_log2
    M = sat_max(bits)
    s = np.asarray(scale, dtype=dtype).reshape(-1, 1)
    step = (s + s) / dtype(2 * M)
    q = step / dtype(W)
    a = (np.asarray(A).astype(np.int64) - M).reshape(-1, c).astype(dtype)
    yhat = a * q
    return T.rht_inverse(yhat.reshape(-1), n, chunk_log2, seed, dtype=dtype, g0=g0)


def sat_pipeline(xs, chunk_log2, seed, bits, dtype=np.float64, bf16=False, g0=0):
    """Rotation and shared scale as in the exact-sum path, then S1-S4."""
    W = len(xs)
    n = len(xs[0])
    ys = [T.rht_forward(x, chunk_log2, seed, dtype=dtype, bf16=bf16, g0=g0) for x in xs]
    scale = T.scale_reduce(np.stack([T.chunk_absmax(y, chunk_log2) for y in ys]))
    idx = [sat_quantize(y, scale, chunk_log2, w, seed, bits, dtype=dtype, g0=g0) for w, y in enumerate(ys)]
    payloads = [T.pack(i, bits) for i in idx]
    A, clipped = sat_aggregate(payloads, bits, count=idx[0].size)
    out = sat_decode(A, scale, W, n, chunk_log2, seed, bits, dtype=dtype, g0=g0)
    return dict(y=ys, scale=scale, idx=idx, payloads=payloads, aggregate=A,
                packed_aggregate=T.pack(A, bits), clipped=clipped, out=out)
