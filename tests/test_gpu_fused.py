"""The batched / fused entry points (one-pass thc_encode_all, thc_aggregate_decode)
against the oracle and against the unfused calls: byte-identical payloads, scales,
sums and outputs."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from synth import generate, workload

from gpu_util import DEV, check_against_oracle, run_path, run_path_fused, sums_to_numpy

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


@pytest.mark.parametrize("l,bits,W,dtype,chunks", [
    (14, 4, 8, torch.bfloat16, 70), (14, 2, 8, torch.bfloat16, 5), (14, 8, 8, torch.bfloat16, 5),
    (14, 4, 8, torch.float32, 9), (14, 8, 3, torch.float32, 4), (14, 2, 1, torch.float32, 3),
    (14, 4, 17, torch.bfloat16, 6), (14, 4, 18, torch.bfloat16, 3), (14, 4, 64, torch.bfloat16, 2),
    (14, 2, 40, torch.float32, 2), (14, 8, 33, torch.bfloat16, 2),
    (14, 8, 1, torch.bfloat16, 3), (14, 8, 1, torch.float32, 2), (14, 8, 2, torch.bfloat16, 2),
    (10, 4, 4, torch.float32, 40), (12, 8, 5, torch.bfloat16, 9), (3, 2, 3, torch.float32, 1000),
    # more than 16 workers (one range word per workgroup) over several rounds of the grid:
    # 25 chunks per round at W = 20, 8 at W = 64
    (14, 4, 20, torch.bfloat16, 60), (14, 2, 64, torch.bfloat16, 20), (14, 8, 33, torch.float32, 31),
])
def test_fused_path_matches_oracle_and_unfused(l, bits, W, dtype, chunks):
    c = 1 << l
    n = chunks * c + (c // 2 + 1 if c > 2 else 1)
    print(f"fused l={l} bits={bits} W={W} dtype={dtype} n={n}", flush=True)
    xs = [_rand(n, dtype, 77 * l + w, scale=10.0 ** (-1 - (w % 4))) for w in range(W)]
    fused = run_path_fused(xs, l, 13, bits)
    check_against_oracle(xs, fused, l, 13, bits)
    plain = run_path(xs, l, 13, bits)
    assert torch.equal(fused["scale"], plain["scale"])
    for a, b in zip(fused["payloads"], plain["payloads"]):
        assert torch.equal(a, b)
    assert torch.equal(fused["sums"], plain["sums"])
    assert torch.equal(fused["out"], plain["out"])
    # sums == NULL is allowed exactly when the fused form applies
    if thc.thc_aggregate_decode_is_fused(W, l, bits):
        nosum = run_path_fused(xs, l, 13, bits, keep_sums=False)
        assert torch.equal(nosum["out"], plain["out"])
    else:
        with pytest.raises(thc.ThcError):
            thc.thc_aggregate_decode(fused["payloads"], fused["scale"], n, l, 13, bits, None,
                                     torch.empty(n, device=DEV))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_scales_outside_and_across_the_folded_range(dtype, bits):
    """Chunks whose scale is tiny (2^-110), huge (2^105) or ordinary side by side: the
    kernels fold the 2^-7 normalisation into the quantizer's constants only where that
    is exact, and both forms must reproduce the oracle bit for bit."""
    l, W, c = 14, 3, 1 << 14
    # (the last three: scales below and around 2^-120, where the reciprocal grid step is not
    # finite in fp32 and the chunk is sent like an all-zero one)
    mags = [2.0 ** -110, 1.0, 2.0 ** 105, 2.0 ** -101, 2.0 ** 99, 2.0 ** -120, 2.0 ** -131, 2.0 ** -124, 2.0 ** -122]
    n = len(mags) * c - 100
    xs = []
    for w in range(W):
        x = _rand(n, torch.float32, 900 + w, scale=1.0)
        for k, m in enumerate(mags):
            x[k * c:(k + 1) * c] *= m
        xs.append(x.to(dtype))
    print(f"extreme scales dtype={dtype} bits={bits}", flush=True)
    fused = run_path_fused(xs, l, 5, bits)
    check_against_oracle(xs, fused, l, 5, bits)
    plain = run_path(xs, l, 5, bits)
    for a, b in zip(fused["payloads"], plain["payloads"]):
        assert torch.equal(a, b)
    assert torch.equal(fused["out"], plain["out"])
    tiny = fused["scale"] < 2.0 ** -120
    assert int(tiny.sum()) >= 1 and float(fused["scale"][tiny].min()) > 0
    per = c * bits // 8
    for k in torch.nonzero(tiny).flatten().tolist():
        assert all(int(p[k * per:(k + 1) * per].max()) == 0 for p in fused["payloads"])


def test_is_fused_predicate():
    assert thc.thc_aggregate_decode_is_fused(8, 14, 4)
    assert thc.thc_aggregate_decode_is_fused(17, 14, 4)
    assert thc.thc_aggregate_decode_is_fused(18, 14, 4) and thc.thc_aggregate_decode_is_fused(64, 14, 4)   # 16-bit lanes
    assert not thc.thc_aggregate_decode_is_fused(65, 14, 4)
    assert thc.thc_aggregate_decode_is_fused(8, 14, 8)
    # one worker of 8-bit payloads has one-byte sums; the fused kernel stores 16-bit lanes
    assert thc.thc_sum_bytes(1, 8) == 1 and not thc.thc_aggregate_decode_is_fused(1, 14, 8)
    assert thc.thc_sum_bytes(2, 8) == 2 and thc.thc_aggregate_decode_is_fused(2, 14, 8)
    assert not thc.thc_aggregate_decode_is_fused(8, 10, 4)
    assert thc.thc_aggregate_decode_is_fused(64, 14, 2)
    assert not thc.thc_aggregate_decode_is_fused(65, 14, 2)


def test_workspace_is_reusable_and_small_inputs_work():
    l, bits, W = 14, 4, 8
    for n in (1, 5000, 1 << 14, (1 << 14) + 1):
        xs = [_rand(n, torch.bfloat16, 3 + w) for w in range(W)]
        a = run_path_fused(xs, l, 5, bits)
        b = run_path(xs, l, 5, bits)
        assert torch.equal(a["out"], b["out"]) and torch.equal(a["sums"], b["sums"])
    # same workspace twice in a row, second call smaller
    n1, n2 = 40 * (1 << 14) + 3, 7 * (1 << 14)
    ws = torch.empty(thc.thc_encode_all_workspace_bytes(W, n1, l), dtype=torch.uint8, device=DEV)
    for n in (n1, n2):
        xs = [_rand(n, torch.bfloat16, 30 + w) for w in range(W)]
        P = thc.thc_num_chunks(n, l)
        pay = [torch.empty(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV) for _ in range(W)]
        sc = torch.empty(P, device=DEV)
        thc.thc_encode_all(xs, l, 6, bits, pay, sc, ws)
        torch.cuda.synchronize()
        assert not thc.thc_encode_all_timed_out(ws)
        ref = run_path(xs, l, 6, bits)
        assert torch.equal(sc, ref["scale"])
        for x, y in zip(pay, ref["payloads"]):
            assert torch.equal(x, y)


def test_expired_wait_sets_the_error_word_and_every_wave_exits():
    """Failure handling forced from the host: with a poll limit of zero the waits
    between workgroups give up at once; the kernel must still finish, and the error
    word reports it.  With the limit restored the same call is correct again."""
    l, bits, W = 14, 4, 8
    n = 600 * (1 << 14)
    xs = [_rand(n, torch.bfloat16, 90 + w) for w in range(W)]
    P = thc.thc_num_chunks(n, l)
    pay = [torch.empty(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV) for _ in range(W)]
    sc = torch.empty(P, device=DEV)
    ws = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
    try:
        thc.thc_set_spin_limit(0)
        thc.thc_encode_all(xs, l, 2, bits, pay, sc, ws)
        torch.cuda.synchronize()            # returns: nothing hangs
        expired = thc.thc_encode_all_timed_out(ws)
    finally:
        thc.thc_set_spin_limit(1 << 22)
    assert expired                           # 4800 items: some wave had to wait at least once
    thc.thc_encode_all(xs, l, 2, bits, pay, sc, ws)
    torch.cuda.synchronize()
    assert not thc.thc_encode_all_timed_out(ws)
    ref = run_path(xs, l, 2, bits)
    assert torch.equal(sc, ref["scale"])
    for x, y in zip(pay, ref["payloads"]):
        assert torch.equal(x, y)


@pytest.mark.parametrize("l,bits,W,dtype,sat", [
    (14, 4, 8, torch.bfloat16, False), (14, 2, 3, torch.float32, False), (14, 8, 17, torch.bfloat16, False),
    (14, 4, 8, torch.bfloat16, True), (10, 4, 4, torch.float32, False),   # (10, ...): unfused fallback
    (14, 4, 5, torch.bfloat16, False), (14, 4, 7, torch.float32, False), (14, 2, 64, torch.bfloat16, False),
    (14, 4, 1, torch.bfloat16, False),
])
def test_cleared_workspace_form_matches_and_leaves_the_workspace_clear(l, bits, W, dtype, sat):
    """thc_encode_all_cleared skips the clearing launch: on a workspace cleared once it must
    give the bytes thc_encode_all gives, call after call, also when the next call is
    smaller, and every byte of the workspace must be zero again after each call."""
    c = 1 << l
    n1, n2 = 37 * c + 11, 6 * c
    ws = torch.full((thc.thc_encode_all_workspace_bytes(W, n1, l),), 0xCD, dtype=torch.uint8, device=DEV)
    thc.thc_workspace_clear(ws)
    plain = thc.thc_sat_encode_all if sat else thc.thc_encode_all
    kept = thc.thc_sat_encode_all_cleared if sat else thc.thc_encode_all_cleared
    for k, n in enumerate((n1, n2, n1)):
        print(f"cleared l={l} bits={bits} W={W} dtype={dtype} sat={sat} n={n}", flush=True)
        xs = [_rand(n, dtype, 500 + 10 * k + w, scale=10.0 ** (-1 - (w % 3))) for w in range(W)]
        P = thc.thc_num_chunks(n, l)
        nb = thc.thc_payload_bytes(n, l, bits)
        got = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
        ref = [torch.full((nb,), 0x55, dtype=torch.uint8, device=DEV) for _ in range(W)]
        sc_got, sc_ref = torch.empty(P, device=DEV), torch.empty(P, device=DEV)
        kept(xs, l, 40 + k, bits, got, sc_got, ws)
        torch.cuda.synchronize()
        assert int(ws.count_nonzero()) == 0, "the workspace did not come back clear"
        ws2 = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
        plain(xs, l, 40 + k, bits, ref, sc_ref, ws2)
        torch.cuda.synchronize()
        assert torch.equal(sc_got, sc_ref)
        for x, y in zip(got, ref):
            assert torch.equal(x, y)


def test_cleared_form_after_an_expired_wait_needs_a_new_clear():
    """A time-out (forced from the host) is reported in the first word; the workspace is
    then no longer clear, and clearing it makes the next call good again."""
    l, bits, W = 14, 4, 8
    n = 600 * (1 << 14)
    xs = [_rand(n, torch.bfloat16, 190 + w) for w in range(W)]
    P = thc.thc_num_chunks(n, l)
    pay = [torch.empty(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV) for _ in range(W)]
    sc = torch.empty(P, device=DEV)
    ws = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
    thc.thc_workspace_clear(ws)
    try:
        thc.thc_set_spin_limit(0)
        thc.thc_encode_all_cleared(xs, l, 2, bits, pay, sc, ws)
        torch.cuda.synchronize()
    finally:
        thc.thc_set_spin_limit(1 << 22)
    assert thc.thc_encode_all_timed_out(ws)
    thc.thc_workspace_clear(ws)
    thc.thc_encode_all_cleared(xs, l, 2, bits, pay, sc, ws)
    torch.cuda.synchronize()
    assert not thc.thc_encode_all_timed_out(ws) and int(ws.count_nonzero()) == 0
    ref = run_path(xs, l, 2, bits)
    assert torch.equal(sc, ref["scale"])
    for x, y in zip(pay, ref["payloads"]):
        assert torch.equal(x, y)


def test_fused_on_full_1p3b_bucket_sampled_chunks():
    wl = workload("gpt_1p3b")
    for k, n in enumerate((wl.buckets()[0][1], wl.buckets()[-1][1])):
        xs = [generate(wl, w, DEV, max_elems=n) for w in range(wl.W)]
        got = run_path_fused(xs, 14, 21 + k, 4, keep_sums=(k == 0))
        P = O.num_chunks(n, 14)
        rng = np.random.default_rng(k)
        chunks = sorted({0, P - 1, P // 2} | set(rng.integers(0, P, size=128).tolist()))
        check_against_oracle(xs, got, 14, 21 + k, 4, chunks=chunks)
        del xs, got
