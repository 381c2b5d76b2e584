"""Min/max-range variant on the GPU against its oracle: ranges, payloads and sums
bit-exact; fp32 output bit-identical to the fp32 canonical order and within 1e-5 relative
L2 of the float64 definition fed the same sums and ranges; bf16 output bit-exact."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from oracle import thc_minmax as M
from synth import to_numpy_bits

from gpu_util import DEV, sums_to_numpy

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3, shift=0.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale + shift).to(dtype)


def run_minmax(xs, l, seed, bits, rotate, out_dtype):
    W, n = len(xs), xs[0].numel()
    P = thc.thc_num_chunks(n, l)
    ranges_all = torch.full((W * P * 2,), float("nan"), device=DEV)
    rng = torch.full((P * 2,), float("nan"), device=DEV)
    nb = thc.thc_payload_bytes(n, l, bits)
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sb = thc.thc_sum_bytes(W, bits)
    sums = torch.full((P << l,), 77, dtype=torch.uint8 if sb == 1 else torch.int16, device=DEV)
    out = torch.zeros(n, dtype=out_dtype, device=DEV)
    for w in range(W):
        thc.thc_chunk_minmax(xs[w], l, seed, rotate, ranges_all[2 * w * P:2 * (w + 1) * P])
    thc.thc_range_reduce(ranges_all, W, P, rng)
    for w in range(W):
        thc.thc_encode_minmax(xs[w], l, seed, w, bits, rotate, rng, payloads[w])
    thc.thc_aggregate(payloads, n, l, bits, sums)
    thc.thc_decode_minmax(sums, rng, W, n, l, seed, bits, rotate, out)
    torch.cuda.synchronize()
    return dict(ranges_all=ranges_all.view(W, P, 2), range=rng.view(P, 2), payloads=payloads, sums=sums, out=out)


@pytest.mark.parametrize("l,bits,W,dtype,chunks,rotate,out_dtype", [
    (14, 4, 4, torch.bfloat16, 5, True, torch.float32), (14, 4, 3, torch.float32, 3, True, torch.float32),
    (14, 8, 2, torch.bfloat16, 2, True, torch.float32), (14, 2, 18, torch.float32, 2, True, torch.float32),
    (14, 4, 4, torch.bfloat16, 3, False, torch.float32), (14, 4, 4, torch.float32, 3, True, torch.bfloat16),
    (14, 4, 3, torch.bfloat16, 2, False, torch.bfloat16),
    (10, 4, 4, torch.float32, 40, True, torch.float32), (10, 8, 3, torch.bfloat16, 17, False, torch.float32),
    (3, 2, 3, torch.float32, 1000, True, torch.bfloat16), (6, 4, 5, torch.float32, 300, False, torch.bfloat16),
])
def test_minmax_path_matches_oracle(l, bits, W, dtype, chunks, rotate, out_dtype):
    c = 1 << l
    n = chunks * c + (c // 2 + 1 if c > 2 else 1)
    print(f"minmax l={l} bits={bits} W={W} dtype={dtype} n={n} rotate={rotate} out={out_dtype}", flush=True)
    # a shift makes the unrotated data (and, through the signs, the rotated data) asymmetric
    xs = [_rand(n, dtype, 13 * l + w, scale=10.0 ** (-2 - (w % 3)), shift=3e-3) for w in range(W)]
    got = run_minmax(xs, l, 17, bits, rotate, out_dtype)
    bf16 = dtype == torch.bfloat16
    out_bf16 = out_dtype == torch.bfloat16
    ref = M.pipeline_minmax([to_numpy_bits(x) for x in xs], l, 17, bits, rotate=rotate, dtype=np.float32,
                            bf16=bf16, out_bf16=out_bf16)
    assert (got["ranges_all"].cpu().numpy() == ref["ranges_all"]).all(), "per-worker ranges differ"
    assert (got["range"].cpu().numpy() == ref["range"]).all(), "shared ranges differ"
    for w in range(W):
        same = got["payloads"][w].cpu().numpy() == ref["payloads"][w]
        assert same.all(), f"payload {w} differs at bytes {np.flatnonzero(~same)[:8]}"
    assert (sums_to_numpy(got["sums"]) == ref["sums"]).all()
    if out_bf16:
        assert (got["out"].view(torch.int16).cpu().numpy().view(np.uint16) == ref["out"]).all()
    else:
        out = got["out"].cpu().numpy()
        assert (out == ref["out"]).all(), "output differs from the fp32 canonical order"
        d64 = M.decode_minmax(ref["sums"], ref["range"].astype(np.float64), W, n, l, 17, bits, rotate)
        assert np.linalg.norm(out - d64) <= 1e-5 * np.linalg.norm(d64)


def test_minmax_with_symmetric_range_equals_the_symmetric_path():
    """Feeding (-s, +s) as the range describes the same grid as thc_encode's; the two
    formulas round in different places, so a handful of indices per million may differ
    by one where the pre-rounding value is an integer to within rounding."""
    l, bits, W = 14, 4, 3
    n = 3 << l
    xs = [_rand(n, torch.bfloat16, 50 + w) for w in range(W)]
    P = n >> l
    absmax = torch.empty(W * P, device=DEV)
    scale = torch.empty(P, device=DEV)
    for w in range(W):
        thc.thc_chunk_absmax(xs[w], l, 3, absmax[w * P:(w + 1) * P])
    thc.thc_scale_reduce(absmax, W, P, scale)
    rng = torch.stack([-scale, scale], dim=1).reshape(-1).contiguous()
    nb = thc.thc_payload_bytes(n, l, bits)
    for w in range(W):
        a = torch.empty(nb, dtype=torch.uint8, device=DEV)
        b = torch.empty(nb, dtype=torch.uint8, device=DEV)
        thc.thc_encode(xs[w], l, 3, w, bits, scale, a)
        thc.thc_encode_minmax(xs[w], l, 3, w, bits, True, rng, b)
        ia = O.unpack(a.cpu().numpy(), bits).astype(int)
        ib = O.unpack(b.cpu().numpy(), bits).astype(int)
        assert (ia != ib).sum() <= 3
        assert np.abs(ia - ib).max() <= 1


def test_minmax_all_equal_chunk_decodes_to_the_constant():
    l, bits, W = 10, 4, 2
    n = 2 << l
    xs = [torch.full((n,), 0.375, device=DEV) for _ in range(W)]
    got = run_minmax(xs, l, 0, bits, False, torch.float32)
    assert (got["range"].cpu().numpy() == 0.375).all()
    for p in got["payloads"]:
        assert (p == 0).all()
    assert (got["out"] == 0.375).all()


@pytest.mark.parametrize("rotate", [True, False])
def test_minmax_coordinates_beyond_2_to_32(rotate):
    """Min/max variant with global indices past 2^32, chunks sampled around the boundary
    and at the ragged end."""
    l, bits, W = 14, 4, 2
    c = 1 << l
    n = (1 << 32) + 2 * c + 55
    g = torch.Generator(device=DEV)
    g.manual_seed(9)
    block = (torch.randn(1 << 24, generator=g, device=DEV) * 1e-3 + 2e-3).to(torch.bfloat16)
    xs = []
    for w in range(W):
        x = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        full = n // block.numel()
        x[:full * block.numel()].view(full, -1).copy_(block.roll(31 * w + 2).unsqueeze(0).expand(full, -1))
        x[full * block.numel():] = block[:n - full * block.numel()]
        xs.append(x)
    print(f"minmax large n={n} rotate={rotate}", flush=True)
    got = run_minmax(xs, l, 4, bits, rotate, torch.float32)
    P = thc.thc_num_chunks(n, l)
    edge = (1 << 32) >> l
    for p in (0, edge - 1, edge, edge + 1, P - 2, P - 1):
        g0 = p * c
        ln = min(n, g0 + c) - g0
        ref = M.pipeline_minmax([to_numpy_bits(x[g0:g0 + ln]) for x in xs], l, 4, bits, rotate=rotate,
                                dtype=np.float32, bf16=True, g0=g0)
        assert (got["range"][p].cpu().numpy() == ref["range"][0]).all(), p
        b0, b1 = g0 * bits // 8, (g0 + c) * bits // 8
        for w in range(W):
            assert (got["payloads"][w][b0:b1].cpu().numpy() == ref["payloads"][w]).all(), (p, w)
        assert (sums_to_numpy(got["sums"][g0:g0 + c]) == ref["sums"]).all(), p
        assert (got["out"][g0:g0 + ln].cpu().numpy() == ref["out"]).all(), p
