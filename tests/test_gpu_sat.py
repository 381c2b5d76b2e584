"""Saturation-based aggregation on the GPU against its oracle: payloads, packed
aggregate and overflow count bit-exact, decoded output within 1e-5 relative L2 of the
float64 definition fed the same aggregate and scales; fused and unfused forms identical."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from oracle import thc_sat as S
from synth import generate, to_numpy_bits, workload

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


def run_sat(xs, l, seed, bits, fused_encode, fused_decode, keep_aggregate=True):
    W, n = len(xs), xs[0].numel()
    P = thc.thc_num_chunks(n, l)
    nb = thc.thc_payload_bytes(n, l, bits)
    scale = torch.full((P,), -1.0, device=DEV)
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    aggregate = torch.full((nb,), 0x55, dtype=torch.uint8, device=DEV)
    overflow = torch.zeros(1, dtype=torch.int64, device=DEV)
    out = torch.full((n,), float("nan"), device=DEV)
    if fused_encode:
        ws = torch.full((thc.thc_encode_all_workspace_bytes(W, n, l),), 0xFF, dtype=torch.uint8, device=DEV)
        thc.thc_sat_encode_all(xs, l, seed, bits, payloads, scale, ws)
    else:
        absmax = torch.empty(W * P, device=DEV)
        for w in range(W):
            thc.thc_chunk_absmax(xs[w], l, seed, absmax[w * P:(w + 1) * P])
        thc.thc_scale_reduce(absmax, W, P, scale)
        for w in range(W):
            thc.thc_sat_encode(xs[w], l, seed, w, bits, scale, payloads[w])
    if fused_decode:
        thc.thc_sat_aggregate_decode(payloads, scale, n, l, seed, bits,
                                     aggregate if keep_aggregate else None, overflow, out)
    else:
        thc.thc_sat_aggregate(payloads, n, l, bits, aggregate, overflow)
        thc.thc_sat_decode(aggregate, scale, W, n, l, seed, bits, out)
    torch.cuda.synchronize()
    if fused_encode:
        assert not thc.thc_encode_all_timed_out(ws)
    return dict(scale=scale, payloads=payloads, aggregate=aggregate if keep_aggregate else None,
                overflow=int(overflow.item()), out=out)


def check_sat(xs, got, l, seed, bits):
    W, n = len(xs), xs[0].numel()
    bf16 = xs[0].dtype == torch.bfloat16
    ref = S.sat_pipeline([to_numpy_bits(x) for x in xs], l, seed, bits, dtype=np.float32, bf16=bf16)
    assert (got["scale"].cpu().numpy() == ref["scale"]).all(), "scale differs"
    for w in range(W):
        same = got["payloads"][w].cpu().numpy() == ref["payloads"][w]
        assert same.all(), f"payload of worker {w} differs at bytes {np.flatnonzero(~same)[:8]}"
    if got["aggregate"] is not None:
        same = got["aggregate"].cpu().numpy() == ref["packed_aggregate"]
        assert same.all(), f"aggregate differs at bytes {np.flatnonzero(~same)[:8]}"
    assert got["overflow"] == int(ref["clipped"].sum()), "overflow count differs"
    d64 = S.sat_decode(ref["aggregate"], ref["scale"].astype(np.float64), W, n, l, seed, bits)
    out = got["out"].cpu().numpy()
    nrm = np.linalg.norm(d64)
    if nrm == 0:
        assert (out == 0).all()
    else:
        err = np.linalg.norm(out - d64) / nrm
        assert err <= 1e-5, f"decode rel-L2 {err}"
    assert (out == ref["out"]).all(), "decode differs from the fp32 canonical order"
    return ref


@pytest.mark.parametrize("l,bits,W,dtype,chunks", [
    (14, 4, 8, torch.bfloat16, 9), (14, 2, 8, torch.bfloat16, 3), (14, 8, 8, torch.bfloat16, 3),
    (14, 4, 4, torch.float32, 5), (14, 4, 1, torch.float32, 2), (14, 8, 3, torch.float32, 2),
    (14, 4, 64, torch.bfloat16, 2), (14, 2, 33, torch.float32, 2),
    (10, 4, 4, torch.float32, 40), (12, 8, 5, torch.bfloat16, 9), (3, 2, 3, torch.float32, 1000),
    (7, 4, 8, torch.bfloat16, 129),
    (14, 4, 8, torch.bfloat16, 150), (14, 4, 40, torch.bfloat16, 30),   # several rounds of the persistent grids
])
def test_sat_path_matches_oracle_fused_and_unfused(l, bits, W, dtype, chunks):
    c = 1 << l
    n = chunks * c + (c // 2 + 1 if c > 2 else 1)
    print(f"sat l={l} bits={bits} W={W} dtype={dtype} n={n}", flush=True)
    # correlated workers (a common component) so that clipping really happens
    common = _rand(n, torch.float32, 5 * l, scale=1e-3)
    xs = [(0.7 * common + _rand(n, torch.float32, 31 * l + w, scale=1e-3)).to(dtype) for w in range(W)]
    plain = run_sat(xs, l, 21, bits, fused_encode=False, fused_decode=False)
    ref = check_sat(xs, plain, l, 21, bits)
    if W >= 4 and bits <= 4:
        assert ref["clipped"].any(), "the case should exercise clipping"
    fused = run_sat(xs, l, 21, bits, fused_encode=True, fused_decode=True)
    assert torch.equal(fused["scale"], plain["scale"])
    for a, b in zip(fused["payloads"], plain["payloads"]):
        assert torch.equal(a, b)
    assert torch.equal(fused["aggregate"], plain["aggregate"])
    assert fused["overflow"] == plain["overflow"]
    assert torch.equal(fused["out"], plain["out"])
    if thc.thc_sat_aggregate_decode_is_fused(W, l, bits):
        lean = run_sat(xs, l, 21, bits, fused_encode=True, fused_decode=True, keep_aggregate=False)
        assert torch.equal(lean["out"], plain["out"]) and lean["overflow"] == plain["overflow"]


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_sat_all_zero_chunks_get_the_centre_index(bits, dtype):
    """A chunk that is zero for every worker has scale 0; on the signed grid its index is
    the centre M (z = 0), through thc_sat_encode and through thc_sat_encode_all alike, and it
    decodes to exactly 0.  Chunks zero for one worker only go through the ordinary rule."""
    l, c, W = 14, 1 << 14, 5
    n = 4 * c + 9
    M = thc.thc_sat_max(bits)
    xs = [_rand(n, dtype, 300 + w) for w in range(W)]
    for x in xs:
        x[:c] = 0
        x[2 * c:3 * c] = 0
    xs[1][c:2 * c] = 0
    for fused in (False, True):
        print(f"sat zero chunks bits={bits} dtype={dtype} fused={fused}", flush=True)
        got = run_sat(xs, l, 9, bits, fused_encode=fused, fused_decode=fused)
        check_sat(xs, got, l, 9, bits)
        assert got["scale"][0].item() == 0 and got["scale"][2].item() == 0
        per = 8 // bits
        centre = sum(M << (bits * j) for j in range(per))           # a byte full of index M
        for p in got["payloads"]:
            assert (p[: c * bits // 8] == centre).all()
            assert (p[2 * c * bits // 8: 3 * c * bits // 8] == centre).all()
        assert (got["out"][:c] == 0).all() and (got["out"][2 * c:3 * c] == 0).all()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_sat_scales_too_small_for_the_reciprocal_step(bits, dtype):
    """Chunks whose scale is below and around 2^-120 (the reciprocal grid step is not finite
    in fp32 below that): sent like all-zero chunks, the centre index everywhere; every form
    against the oracle."""
    l, c, W = 14, 1 << 14, 3
    n = 4 * c
    M = thc.thc_sat_max(bits)
    xs = []
    for w in range(W):
        x = _rand(n, torch.float32, 700 + w, scale=1.0)
        x[:c] *= 2.0 ** -131
        x[c:2 * c] *= 2.0 ** -123
        x[2 * c:3 * c] *= 2.0 ** -121
        xs.append(x.to(dtype))
    for fused in (False, True):
        print(f"sat tiny scales bits={bits} dtype={dtype} fused={fused}", flush=True)
        got = run_sat(xs, l, 3, bits, fused_encode=fused, fused_decode=fused)
        check_sat(xs, got, l, 3, bits)
        assert 0 < got["scale"][0].item() < 2.0 ** -121
        centre = sum(M << (bits * j) for j in range(8 // bits))
        for p in got["payloads"]:
            assert (p[: c * bits // 8] == centre).all()


def test_sat_without_clipping_equals_exact_sum_decode():
    """Small, cancelling values: no Sat step clips, so the saturated aggregate is the
    exact integer sum and the decoded mean equals the exact-sum decode of the same
    payloads on the (2M+1)-point grid up to rounding."""
    l, bits, W = 14, 8, 2
    n = 3 << l
    x = _rand(n, torch.float32, 3)
    xs = [x, -x]
    got = run_sat(xs, l, 4, bits, fused_encode=True, fused_decode=True)
    ref = check_sat(xs, got, l, 4, bits)
    assert got["overflow"] == 0 and not ref["clipped"].any()
    M = S.sat_max(bits)
    a = ref["aggregate"].astype(int) - M
    z = [i.astype(int) - M for i in ref["idx"]]
    assert (a == z[0] + z[1]).all()


def test_sat_worker_limit_and_null_aggregate():
    l, bits, n = 14, 4, 1 << 14
    pay = [torch.zeros(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV) for _ in range(65)]
    scale = torch.ones(1, device=DEV)
    out = torch.empty(n, device=DEV)
    with pytest.raises(thc.ThcError):
        thc.thc_sat_aggregate_decode(pay, scale, n, l, 0, bits, None, None, out)
    with pytest.raises(thc.ThcError):      # not fused for chunk 2^10: the aggregate buffer is required
        thc.thc_sat_aggregate_decode(pay[:4], torch.ones(16, device=DEV), n, 10, 0, bits, None, None, out)


def test_sat_on_headline_bucket_sampled_chunks():
    """One full 1.3B-workload bucket (W = 8, bf16, b = 4) in the launch configuration the
    benchmark times; the oracle checks sampled chunks (chunks are independent)."""
    wl = workload("gpt_1p3b")
    l, bits, W = wl.chunk_log2, 4, wl.W
    n = wl.buckets()[0][1]
    xs = [generate(wl, w, torch.device(DEV), max_elems=n) for w in range(W)]
    got = run_sat(xs, l, 0, bits, fused_encode=True, fused_decode=True)
    c = 1 << l
    P = n // c
    rng = np.random.default_rng(0)
    total_clipped = 0
    for p in sorted(set([0, P - 1] + rng.integers(0, P, size=6).tolist())):
        hx = [to_numpy_bits(x[p * c:(p + 1) * c]) for x in xs]
        ref = S.sat_pipeline(hx, l, 0, bits, dtype=np.float32, bf16=True, g0=p * c)
        b0, b1 = p * c * bits // 8, (p + 1) * c * bits // 8
        for w in range(W):
            assert (got["payloads"][w][b0:b1].cpu().numpy() == ref["payloads"][w]).all(), f"chunk {p}"
        assert (got["aggregate"][b0:b1].cpu().numpy() == ref["packed_aggregate"]).all(), f"chunk {p}"
        assert (got["out"][p * c:(p + 1) * c].cpu().numpy() == ref["out"]).all(), f"chunk {p}"
        total_clipped += int(ref["clipped"].sum())
    assert 0 <= got["overflow"] <= n
    print(f"overflow rate on the bucket: {got['overflow'] / n:.4f}", flush=True)


def test_sat_coordinates_beyond_2_to_32():
    """Saturating variant with global indices past 2^32 (both encode forms, both
    aggregate + decode forms), chunks sampled around the boundary and at the ragged end.
    The overflow count, which covers every coordinate, is compared between the forms."""
    l, bits, W = 14, 4, 2
    c = 1 << l
    n = (1 << 32) + 2 * c + 321
    g = torch.Generator(device=DEV)
    g.manual_seed(8)
    block = (torch.randn(1 << 24, generator=g, device=DEV) * 1e-3).to(torch.bfloat16)
    xs = []
    for w in range(W):
        x = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        full = n // block.numel()
        x[:full * block.numel()].view(full, -1).copy_(block.roll(77 * w + 5).unsqueeze(0).expand(full, -1))
        x[full * block.numel():] = block[:n - full * block.numel()]
        xs.append(x)
    P = thc.thc_num_chunks(n, l)
    edge = (1 << 32) >> l
    results = []
    for fused in (True, False):
        print(f"sat large n={n} fused={fused}", flush=True)
        got = run_sat(xs, l, 6, bits, fused, fused)
        for p in (0, edge - 1, edge, edge + 1, P - 2, P - 1):
            g0 = p * c
            ln = min(n, g0 + c) - g0
            ref = S.sat_pipeline([to_numpy_bits(x[g0:g0 + ln]) for x in xs], l, 6, bits, dtype=np.float32,
                                 bf16=True, g0=g0)
            assert float(got["scale"][p]) == float(ref["scale"][0])
            b0, b1 = g0 * bits // 8, (g0 + c) * bits // 8
            for w in range(W):
                assert (got["payloads"][w][b0:b1].cpu().numpy() == ref["payloads"][w]).all(), (p, w)
            assert (got["aggregate"][b0:b1].cpu().numpy() == ref["packed_aggregate"]).all(), p
            assert (got["out"][g0:g0 + ln].cpu().numpy() == ref["out"]).all(), p
        results.append(got)
    a, b = results
    assert a["overflow"] == b["overflow"]
    assert torch.equal(a["aggregate"], b["aggregate"]) and torch.equal(a["out"], b["out"])
