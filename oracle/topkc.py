"""CPU oracle of TopK Chunked (TopKC), the all-reduce-compatible sparsification of the
paper's TopK case study ("Our proposed improvement: Chunks", design changes 1 and 2).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

What the paper fixes: the gradient is cut into ceil(d / C) chunks of C coordinates; every
worker computes the squared L2 norm of each chunk, in half precision; these are summed
over workers with an all-reduce, s_p = sum_i ||c_p^(i)||^2; all workers pick the J chunks
with the largest s_p; the selected chunks are summed with an all-reduce in half precision
(FP16); the cost is b = 16 (J C / d + 1 / C) bits per coordinate.

Readings where it is silent:
  T1  The gradient is zero-padded to a multiple of C.  C is a power of two, 8 <= C <= 1024.
  T2  Norm of one chunk: x widened to fp32, squares rounded to fp32, summed in fp32 as a
      balanced tree over adjacent pairs ((x0^2 + x1^2) + (x2^2 + x3^2)) + ..., the result
      rounded to fp16 (nearest even; overflow gives inf, tiny values go subnormal or 0).
  T3  An fp16 all-reduce adds fp16 numbers: s_p accumulates in fp16 in worker order
      0, 1, ..., W-1, every partial sum rounded to fp16.
  T4  Selection: the J largest s_p; equal values are taken lowest chunk index first; the
      selected indices are listed in ascending order.
  T5  Selected chunks: every worker's values rounded to fp16, summed in fp16 in worker
      order (what the FP16 all-reduce of the sparsified gradients computes).
  T6  Decode: the estimate of the MEAN gradient is float(sum) / W on the selected chunks
      and 0 elsewhere.
"""

import numpy as np

from . import thc as T


def num_chunks(d, C):
    return (d + C - 1) // C


def bits_per_coordinate(J, C, d):
    """The paper's cost formula b = 16 (J C / d + 1 / C)."""
    return 16.0 * (J * C / d + 1.0 / C)


def _padded_fp32(x, C, bf16):
    x = T._widen(x, bf16, np.float32)
    P = num_chunks(len(x), C)
    a = np.zeros(P * C, dtype=np.float32)
    a[:len(x)] = x
    return a.reshape(P, C)


def chunk_norms(x, C, bf16=False):
    """T2.  Returns P fp16 values."""
    a = _padded_fp32(x, C, bf16)
    sq = a * a                                     # fp32, one rounding each
    while sq.shape[1] > 1:
        sq = sq[:, 0::2] + sq[:, 1::2]             # adjacent pairs, fp32
    return sq[:, 0].astype(np.float16)


def sum_fp16(arrays):
    """T3 / T5: fp16 accumulation in list order, one rounding per addition."""
    acc = np.asarray(arrays[0], dtype=np.float16).copy()
    for a in arrays[1:]:
        acc = (acc.astype(np.float32) + np.asarray(a, dtype=np.float16).astype(np.float32)).astype(np.float16)
    return acc


def select(s, J):
    """T4.  s: P non-negative fp16 values.  Returns J chunk indices, ascending."""
    s = np.asarray(s, dtype=np.float16)
    assert 0 < J <= s.size
    order = np.lexsort((np.arange(s.size), -s.astype(np.float64)))   # value descending, index ascending
    return np.sort(order[:J]).astype(np.uint32)


def gather_sum(xs, C, indices, bf16=False):
    """T5.  Returns (J, C) fp16: the fp16 sum over workers of the selected chunks."""
    idx = np.asarray(indices, dtype=np.int64)
    parts = [_padded_fp32(x, C, bf16)[idx].astype(np.float16) for x in xs]
    return sum_fp16(parts)


def scatter_mean(values, indices, C, W, d):
    """T6.  Dense fp32 estimate of the mean gradient (d coordinates)."""
    P = num_chunks(d, C)
    out = np.zeros((P, C), dtype=np.float32)
    out[np.asarray(indices, dtype=np.int64)] = np.asarray(values, dtype=np.float16).astype(np.float32) / np.float32(W)
    return out.reshape(-1)[:d]


def pipeline(xs, C, J, bf16=False):
    W, d = len(xs), len(xs[0])
    norms = [chunk_norms(x, C, bf16) for x in xs]
    s = sum_fp16(norms)
    idx = select(s, J)
    vals = gather_sum(xs, C, idx, bf16)
    out = scatter_mean(vals, idx, C, W, d)
    return dict(norms=norms, s=s, indices=idx, values=vals, out=out)
