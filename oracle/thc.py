"""Step-by-step CPU oracle of the chunked randomized-Hadamard quantization path.

TEST INFRASTRUCTURE ONLY (see the package docstring): the product never imports
this file.  Everything is plain NumPy, one obvious operation per line, no
blocking or fusion, so that it can be checked against the paper by eye.

What the paper fixes (THC Quantization subsection):
  * "Background and issues": gradients are rotated by a Randomized Hadamard
    Transform, then each coordinate is stochastically rounded to one of the two
    nearest points of an evenly spaced grid whose points are the q-bit integers
    0 .. 2^q - 1; the aggregate of coordinate p is the integer sum over workers
    of the quantized values, held in b >= q bits so it cannot overflow.
  * "Partial rotation": stopping the transform after l' <= l iterations equals
    rotating each 2^l'-sized chunk on its own; afterwards the value range is
    taken per chunk so a large coordinate only hurts precision locally.
  * Notation table: q, l, l', padding of the gradient to a power of two.
The receiver side (dequantize, rotate back, average) is implied by these.

What the paper leaves open, and the reading taken here (the same readings are
implemented, independently, by the GPU library):
  R1  Hadamard ordering / normalisation: Sylvester (natural) order,
      H[i][j] = (-1)^popcount(i & j), orthonormal factor 1/sqrt(c) on both
      directions, butterfly stages from stride 1 up to c/2 (the recursion
      H_k = H_1 (x) H_{k-1} on neighbouring halves).
  R2  "Randomized": a +-1 diagonal D applied before H, the same for every
      worker (so that rotating commutes with summing over workers), taken from
      Philox4x32-10 by the coordinate's global index.
  R3  Range: one symmetric range [-s_p, +s_p] per chunk, s_p the largest
      |rotated value| of chunk p over ALL workers (integer sums are only
      decodable when every worker used the same grid).
  R4  Levels: L + 1 = 2^b grid points, index 0 at -s_p and index L at +s_p.
  R5  Rounding: idx = floor(v + u), v = y * inv + L/2 the position in grid units
      (inv = L / (2 s_p)), u uniform in (0,1) built from RBITS random bits, centred:
      u = (r + 0.5) / 2^RBITS.  The fp32 mode evaluates v + u in the order that keeps
      it within 1e-6 * max(1, |t|) of the float64 definition for every grid size
      (see grid_position_plus_noise): fma(y, inv, L/2 + u) for grids of up to 32
      points (L/2 + u is exact), fma(y + s_p, inv, u) for larger ones; an all-zero
      chunk has index 0 everywhere.
  R6  Decode returns the estimate of the workers' MEAN gradient.
  R7  All-zero chunk (s_p = 0): every index is 0 and it decodes to exactly 0.
      The same indices for a chunk whose range is too small for the arithmetic: the rule
      needs the reciprocal grid step L / (2 s_p), which is not finite in binary32 once
      2 s_p falls below about 2^-120 (L = 255); a chunk with 2 s_p < MIN_RANGE = 2^-119 is
      therefore quantized like an all-zero chunk, in both modes.  Its scale is kept, so
      it decodes to -s_p per rotated coordinate: an error of at most 2^-119.
  R8  Padding: zeros up to a multiple of the chunk only.

Two arithmetic modes with identical logic: dtype=np.float64 is the definition;
dtype=np.float32 performs every real operation as one separately rounded
IEEE-754 binary32 operation in the order written here (the "canonical order"),
so that a device that does the same operations produces the same bits.
"""

import numpy as np

from .philox import philox4x32_10

#: random bits consumed per coordinate by the stochastic rounding (reading R5)
RBITS = 8
#: smallest width of a chunk's range (2 s_p, or hi - lo on the min/max grid) that is quantized
#: by the rule; narrower ranges are treated like an empty one (reading R7)
MIN_RANGE = 2.0 ** -119
#: fourth counter word that separates the two uses of the generator
TAG_SIGN = 0x5349474E
TAG_ROUND = 0x524F554E

_M32 = 0xFFFFFFFF


# --------------------------------------------------------------------------- sizes
def num_chunks(n, chunk_log2):
    """Chunks of 2^l' coordinates needed to cover n (partial rotation: one
    independent rotation per chunk)."""
    c = 1 << chunk_log2
    return (n + c - 1) // c


def payload_bytes(n, chunk_log2, bits):
    """Bytes of one worker's packed q-bit payload (padded chunks included; a last
    partial byte, possible only for 2 coordinates of 2 bits, is counted whole)."""
    return (num_chunks(n, chunk_log2) * (1 << chunk_log2) * bits + 7) // 8


def sum_dtype(W, bits):
    """Narrowest unsigned type that holds W * (2^bits - 1): the widened
    aggregate of the "simple adaptation" (b >= q bits so sums cannot overflow)."""
    top = W * ((1 << bits) - 1)
    if top <= 0xFF:
        return np.uint8
    if top <= 0xFFFF:
        return np.uint16
    raise ValueError("W * (2^bits - 1) does not fit 16 bits")


# ------------------------------------------------------------------ random streams
def sign_bits(g0, count, seed):
    """Reading R2.  Boolean array, True where D_gg = -1, for global indices
    g0 .. g0+count-1.  Bit (g mod 32) of word ((g div 32) mod 4) of the Philox
    block with counter (lo32(g div 128), hi32(g div 128), 0, TAG_SIGN) and key
    (lo32(seed), hi32(seed))."""
    g = np.arange(g0, g0 + count, dtype=np.uint64)
    block = g // np.uint64(128)
    first = int(g0) // 128
    last = (int(g0) + max(count, 1) - 1) // 128
    ids = np.arange(first, last + 1, dtype=np.uint64)
    words = philox4x32_10(ids & np.uint64(_M32), ids >> np.uint64(32), 0, TAG_SIGN,
                          seed & _M32, (seed >> 32) & _M32)          # (blocks, 4)
    w = words[(block - np.uint64(first)).astype(np.int64),
              ((g // np.uint64(32)) % np.uint64(4)).astype(np.int64)]
    bit = (w >> (g % np.uint64(32)).astype(np.uint32)) & np.uint32(1)
    return bit.astype(bool)


def rounding_fields(g0, count, worker, seed, rbits=RBITS):
    """Reading R5.  The RBITS-bit integers r_g for global indices g0..g0+count-1
    of one worker.  One Philox block with counter (lo32(g div E), hi32(g div E),
    worker, TAG_ROUND), E = 128 / RBITS, serves E consecutive coordinates;
    coordinate g takes field k = g mod E, fields counted low bits first through
    word 0, then word 1, ..."""
    if rbits not in (4, 8, 16, 32):
        raise ValueError("rbits")
    per_block = 128 // rbits
    per_word = 32 // rbits
    g = np.arange(g0, g0 + count, dtype=np.uint64)
    block = g // np.uint64(per_block)
    first = int(g0) // per_block
    last = (int(g0) + max(count, 1) - 1) // per_block
    ids = np.arange(first, last + 1, dtype=np.uint64)
    words = philox4x32_10(ids & np.uint64(_M32), ids >> np.uint64(32), worker, TAG_ROUND,
                          seed & _M32, (seed >> 32) & _M32)
    k = (g % np.uint64(per_block)).astype(np.int64)
    w = words[(block - np.uint64(first)).astype(np.int64), k // per_word].astype(np.uint64)
    shift = (rbits * (k % per_word)).astype(np.uint64)
    return ((w >> shift) & np.uint64((1 << rbits) - 1)).astype(np.uint32)


# ------------------------------------------------------------------------ rotation
def fwht(a):
    """Unnormalised Walsh-Hadamard transform along the last axis, in place,
    Sylvester order, stages h = 1, 2, 4, ... (reading R1).  Every stage replaces
    each pair (a[i], a[i+h]) with (a[i] + a[i+h], a[i] - a[i+h]), one rounded
    operation each in the array's own dtype."""
    c = a.shape[-1]
    assert c & (c - 1) == 0
    h = 1
    while h < c:
        v = a.reshape(-1, c // (2 * h), 2, h)
        lo = v[:, :, 0, :].copy()
        hi = v[:, :, 1, :].copy()
        v[:, :, 0, :] = lo + hi
        v[:, :, 1, :] = lo - hi
        h *= 2
    return a


def _widen(x, bf16, dtype):
    """Inputs are fp32, or bf16 given as their 16-bit patterns (exactly widened)."""
    x = np.asarray(x)
    if bf16:
        assert x.dtype == np.uint16
        x = (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    else:
        assert x.dtype == np.float32 or x.dtype == np.float64
    return x.astype(dtype)


def _inv_sqrt(c, dtype):
    return dtype(1.0 / np.sqrt(np.float64(c)))


def rht_forward(x, chunk_log2, seed, dtype=np.float64, bf16=False, g0=0):
    """y = (1/sqrt(c)) H_c D x per chunk ("Partial rotation": l' stages = each
    2^l' chunk rotated separately).  x holds coordinates g0 .. g0+len(x)-1 of the
    flattened gradient (g0 a multiple of c); zeros are appended up to a whole
    chunk (R8).  Returns chunks*c values."""
    c = 1 << chunk_log2
    assert g0 % c == 0
    n = len(x)
    P = num_chunks(n, chunk_log2)
    a = np.zeros(P * c, dtype=dtype)
    a[:n] = _widen(x, bf16, dtype)
    neg = sign_bits(g0, P * c, seed)
    a[neg] = -a[neg]
    a = fwht(a.reshape(P, c)).reshape(-1)
    a *= _inv_sqrt(c, dtype)
    return a


def rht_inverse(y, n, chunk_log2, seed, dtype=np.float64, g0=0):
    """x = D (1/sqrt(c)) H_c y per chunk (H is symmetric and H H = c I, D D = I,
    so this undoes rht_forward); only the first n coordinates are returned."""
    c = 1 << chunk_log2
    P = num_chunks(n, chunk_log2)
    a = np.array(y, dtype=dtype).reshape(P, c)
    a = fwht(a).reshape(-1)
    a *= _inv_sqrt(c, dtype)
    neg = sign_bits(g0, P * c, seed)
    a[neg] = -a[neg]
    return a[:n]


# --------------------------------------------------------------------------- scale
def chunk_absmax(y, chunk_log2):
    """Per-chunk range after the partial rotation, symmetric reading R3:
    a_p = max_j |y_j| over chunk p."""
    c = 1 << chunk_log2
    return np.abs(y.reshape(-1, c)).max(axis=1)


def scale_reduce(absmax_all):
    """Shared grid (R3): s_p = max over workers of a_p^(w).  absmax_all: (W, P)."""
    return np.max(np.asarray(absmax_all), axis=0)


# ------------------------------------------------------------------------ quantizer
def fma32(a, b, c):
    """Correctly rounded float32 fused multiply-add a * b + c of float32 arrays, built from
    float64 operations.  The product of two float32 numbers is exact in float64; the sum
    p + c is computed with its exact rounding error e (TwoSum), and rounding s = fl64(p + c)
    to float32 gives the right answer unless s sits exactly halfway between two float32
    numbers while e != 0, in which case e decides the direction."""
    a = np.asarray(a, dtype=np.float32).astype(np.float64)
    b = np.asarray(b, dtype=np.float32).astype(np.float64)
    c = np.asarray(c, dtype=np.float32).astype(np.float64)
    a, b, c = np.broadcast_arrays(a, b, c)
    p = a * b
    s = p + c
    bb = s - p                                   # TwoSum (Knuth): e = exact (p + c) - s
    e = (p - (s - bb)) + (c - bb)
    r = s.astype(np.float32)
    r64 = r.astype(np.float64)
    inexact = r64 != s
    if inexact.any():
        toward = np.where(s > r64, np.float32(np.inf), np.float32(-np.inf))
        other = np.nextafter(r, toward)          # the float32 neighbour on the far side of s
        tie = inexact & (np.abs(s - r64) == np.abs(other.astype(np.float64) - s))
        fix = tie & (e != 0)
        if fix.any():
            up = np.maximum(r, other)
            dn = np.minimum(r, other)
            r = np.where(fix, np.where(e > 0, up, dn), r).astype(np.float32)
    return r


#: Largest grid index for which the fp32 mode forms the position with one fused operation
#: from y itself; larger grids (8-bit payloads) take the offset y + s first.
SINGLE_FMA_MAX_LEVELS = 31


def grid_position_plus_noise(y, s, inv, L, u, dtype):
    """t = (position of y on the grid of [-s, s], in grid units) + u.

    float64, the definition:      t = y * inv + L/2 + u.
    float32, the canonical order, chosen by grid size so that t stays within the band
    1e-6 * max(1, |t|) of the definition (the band inside which an index may differ):

      L <= 31 (2- and 4-bit grids):   t = fma(y, inv, L/2 + u)   one rounding; L/2 + u is exact.
          inv = fl(L / (2 s)) carries a relative error of at most 2^-24, which the product
          turns into an ABSOLUTE error of |y * inv| * 2^-24 <= (L/2) 2^-24 in t, plus the final
          rounding |t| 2^-24:  (L/2 + |t|) 2^-24 <= (15.5 + |t|) 6e-8 < 1e-6 max(1, |t|).
      L >= 32 (8-bit grids):          t = fma(fl(y + s), inv, u)  the offset is rounded first.
          With L = 255 the bound above is 7.6e-6 at the low end of the grid (|t| near 1),
          outside the band.  Here every error is relative to the offset value itself:
          |t| (2^-24 + 2^-24 + 2^-24) <= 1.8e-7 |t|.

    tests/test_oracle_quantizer.py measures both claims on 10^7 samples per grid size."""
    if dtype != np.float32:
        return y * inv + dtype(L / 2.0) + u
    if L <= SINGLE_FMA_MAX_LEVELS:
        return fma32(y, inv, np.float32(L / 2.0) + u)      # L/2 + u: exact short binary fraction
    return fma32((y + s).astype(np.float32), inv, u)


def quantize(y, scale, chunk_log2, worker, seed, bits, dtype=np.float64, g0=0,
             rbits=RBITS, return_t=False, r=None):
    """Stochastic rounding onto the 2^bits-point grid of [-s_p, s_p] (THC
    background paragraph: evenly split range, grid points at the boundaries,
    each coordinate rounded to one of its two neighbours; readings R4, R5, R7).

        inv = L / (s_p + s_p)
        t   = y * inv + L/2 + u,  u = (r + 0.5) / 2^RBITS     (position in grid units + noise;
                                  fp32 evaluation order: grid_position_plus_noise)
        idx = min(floor(t), L);   2 s_p < MIN_RANGE (in particular s_p = 0) -> idx = 0

    `r` (tests only) replaces the generator's RBITS-bit integers, so that every
    value of r can be enumerated by brute force.
    """
    c = 1 << chunk_log2
    L = (1 << bits) - 1
    y = np.asarray(y, dtype=dtype).reshape(-1, c)
    s = np.asarray(scale, dtype=dtype).reshape(-1, 1)
    two_s = s + s
    inv = np.zeros_like(two_s)
    nz = two_s >= dtype(MIN_RANGE)
    inv[nz] = dtype(L) / two_s[nz]
    if r is None:
        r = rounding_fields(g0, y.size, worker, seed, rbits)
    r = np.asarray(r).reshape(y.shape)
    u = (r.astype(dtype) + dtype(0.5)) * dtype(2.0 ** -rbits)
    t = grid_position_plus_noise(y, s, inv, L, u, dtype)
    idx = np.minimum(np.floor(t), dtype(L)).astype(np.uint16)
    idx[np.broadcast_to(~nz, idx.shape)] = 0
    idx = idx.reshape(-1)
    if return_t:
        return idx, np.asarray(t, dtype=dtype).reshape(-1)
    return idx


def pack(idx, bits):
    """q-bit payload, little-endian inside each byte: element j of a byte's group
    sits at bit (j * bits) mod 8."""
    idx = np.asarray(idx).astype(np.uint16)
    assert idx.max(initial=0) < (1 << bits)
    if bits == 8:
        return idx.astype(np.uint8)
    per = 8 // bits
    if idx.size % per:
        idx = np.concatenate([idx, np.zeros(per - idx.size % per, dtype=np.uint16)])
    g = idx.reshape(-1, per)
    out = np.zeros(g.shape[0], dtype=np.uint16)
    for j in range(per):
        out |= g[:, j] << np.uint16(j * bits)
    return out.astype(np.uint8)


def unpack(payload, bits):
    payload = np.asarray(payload, dtype=np.uint8)
    if bits == 8:
        return payload.astype(np.uint16)
    per = 8 // bits
    out = np.zeros((payload.size, per), dtype=np.uint16)
    for j in range(per):
        out[:, j] = (payload >> np.uint8(j * bits)) & np.uint8((1 << bits) - 1)
    return out.reshape(-1)


# ----------------------------------------------------------------------- aggregate
def aggregate(payloads, bits, count=None):
    """S_g = sum over workers of idx_g^(w), exact, in the narrowest of u8/u16 that
    cannot overflow ("All-reduce incompatibility": b >= q bits for the sums)."""
    W = len(payloads)
    total = np.zeros(np.asarray(payloads[0]).size * 8 // bits, dtype=np.int64)
    for p in payloads:
        total += unpack(p, bits)
    assert total.max(initial=0) <= W * ((1 << bits) - 1)
    if count is not None:            # drop the unused bits of a last partial byte
        total = total[:count]
    return total.astype(sum_dtype(W, bits))


# -------------------------------------------------------------------------- decode
def decode(sums, scale, W, n, chunk_log2, seed, bits, dtype=np.float64, g0=0):
    """Receiver side (implied by the paper): grid index sums back to values,
    averaged over the W workers (R6), then the inverse rotation.

        step  = (s_p + s_p) / L
        yhat  = S * (step / W) - s_p
        xhat  = D (1/sqrt(c)) H_c yhat,   first n coordinates
    """
    c = 1 << chunk_log2
    L = (1 << bits) - 1
    s = np.asarray(scale, dtype=dtype).reshape(-1, 1)
    step = (s + s) / dtype(L)
    q = step / dtype(W)
    S = np.asarray(sums).reshape(-1, c).astype(dtype)
    yhat = S * q - s
    return rht_inverse(yhat.reshape(-1), n, chunk_log2, seed, dtype=dtype, g0=g0)


# ------------------------------------------------------------------------ whole path
def pipeline(xs, chunk_log2, seed, bits, dtype=np.float64, bf16=False, g0=0, rbits=RBITS):
    """All steps for W workers' gradients xs[w] (equal lengths).  Returns a dict
    with every intermediate so tests can compare stage by stage."""
    W = len(xs)
    n = len(xs[0])
    ys = [rht_forward(x, chunk_log2, seed, dtype=dtype, bf16=bf16, g0=g0) for x in xs]
    absmax = np.stack([chunk_absmax(y, chunk_log2) for y in ys])
    scale = scale_reduce(absmax)
    idx, ts = [], []
    for w, y in enumerate(ys):
        i, t = quantize(y, scale, chunk_log2, w, seed, bits, dtype=dtype, g0=g0,
                        rbits=rbits, return_t=True)
        idx.append(i)
        ts.append(t)
    payloads = [pack(i, bits) for i in idx]
    sums = aggregate(payloads, bits, count=idx[0].size)   # (a last partial byte holds no coordinates)
    out = decode(sums, scale, W, n, chunk_log2, seed, bits, dtype=dtype, g0=g0)
    return dict(y=ys, absmax=absmax, scale=scale, idx=idx, t=ts, payloads=payloads,
                sums=sums, out=out)
