"""The batched entry points (several buckets per launch) against the per-bucket calls:
byte-identical payloads, scales and outputs; error paths."""
import pytest
import torch

import paper_2407_01378_amd as thc

from gpu_util import DEV, check_against_oracle

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


def _make(ns, W, dtype, bits, l=14):
    buckets = []
    for k, n in enumerate(ns):
        xs = [_rand(n, dtype, 1000 * k + w, scale=10.0 ** (-1 - (w % 3))) for w in range(W)] if n else \
             [torch.empty(0, dtype=dtype, device=DEV) for _ in range(W)]
        P = thc.thc_num_chunks(n, l)
        nb = thc.thc_payload_bytes(n, l, bits)
        buckets.append(dict(
            grads=xs, n=n, seed=77 + 3 * k,
            payloads=[torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)],
            scale=torch.full((P,), -1.0, device=DEV),
            out=torch.full((n,), float("nan"), device=DEV)))
    return buckets


@pytest.mark.parametrize("W,dtype,bits,ns", [
    (8, torch.bfloat16, 4, [5 << 14, (3 << 14) + 100, 16384, 700 << 14, 40, (9 << 14) + 8193]),
    (8, torch.bfloat16, 4, [(2 << 14) + 78, 0, 1 << 14]),            # even counts only, an empty bucket
    (3, torch.float32, 8, [(4 << 14) + 5, 6 << 14]),
    (17, torch.bfloat16, 2, [(2 << 14) + 1, 3 << 14, 100]),
    (1, torch.float32, 4, [(70 << 14) + 3]),
    (64, torch.bfloat16, 2, [1 << 14, (1 << 14) + 2]),
    (18, torch.bfloat16, 4, [(2 << 14) + 2, 1 << 14]),               # sums of 18 workers need 16-bit accumulators
    (40, torch.float32, 4, [(1 << 14) + 7]),
])
def test_batched_calls_match_the_per_bucket_calls(W, dtype, bits, ns):
    l = 14
    batch = _make(ns, W, dtype, bits)
    ws = torch.full((thc.thc_batch_workspace_bytes(ns, W, l),), 0xFF, dtype=torch.uint8, device=DEV)
    print(f"batch W={W} dtype={dtype} bits={bits} ns={ns}", flush=True)
    for rep in range(2):                        # the workspace is reusable as it comes back
        thc.thc_encode_all_batch(batch, l, bits, ws)
        thc.thc_aggregate_decode_batch(batch, l, bits, ws)
        torch.cuda.synchronize()
        assert not thc.thc_encode_all_timed_out(ws)
    for k, b in enumerate(batch):
        n = b["n"]
        if n == 0:
            continue
        P = thc.thc_num_chunks(n, l)
        ref_pay = [torch.full_like(p, 0x55) for p in b["payloads"]]
        ref_sc = torch.empty(P, device=DEV)
        ref_out = torch.empty(n, device=DEV)
        w1 = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
        thc.thc_encode_all(b["grads"], l, b["seed"], bits, ref_pay, ref_sc, w1)
        thc.thc_aggregate_decode(ref_pay, ref_sc, n, l, b["seed"], bits, None, ref_out)
        torch.cuda.synchronize()
        assert torch.equal(b["scale"], ref_sc), f"scale of bucket {k}"
        for w in range(W):
            assert torch.equal(b["payloads"][w], ref_pay[w]), f"payload {w} of bucket {k}"
        assert torch.equal(b["out"], ref_out), f"output of bucket {k}"
    # and one bucket element by element against the oracle
    k = 1 if len(ns) > 1 and ns[1] else 0
    if ns[k] <= (9 << 14) + 8193 and W <= 18:
        b = batch[k]
        check_against_oracle(b["grads"], dict(scale=b["scale"], payloads=b["payloads"], sums=None, out=b["out"]),
                             l, b["seed"], bits)


def test_batched_calls_refuse_what_they_do_not_cover():
    l = 14
    batch = _make([1 << 14], 4, torch.float32, 4)
    ws = torch.empty(thc.thc_batch_workspace_bytes([1 << 14], 4, l), dtype=torch.uint8, device=DEV)
    with pytest.raises(thc.ThcError) as e:
        thc.thc_encode_all_batch(batch, 10, 4, ws)
    assert e.value.status == -3
    with pytest.raises(thc.ThcError) as e:
        thc.thc_encode_all_batch(batch, l, 4, ws[:64])
    assert e.value.status == -6
    one = _make([1 << 14], 1, torch.bfloat16, 8)            # one worker of 8-bit payloads: the decode side is not fused
    ws2 = torch.empty(thc.thc_batch_workspace_bytes([1 << 14], 1, l), dtype=torch.uint8, device=DEV)
    thc.thc_encode_all_batch(one, l, 8, ws2)
    with pytest.raises(thc.ThcError) as e:
        thc.thc_aggregate_decode_batch(one, l, 8, ws2)
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert thc.thc_batch_workspace_bytes([1 << 14], 4, 10) == 0


def test_payloads_do_not_depend_on_which_workgroup_takes_which_chunk():
    """Determinism under a permuted workgroup order: the same bucket placed after 0, 1, 7 and
    100 chunks of another bucket in a batched call is handled by other workgroups, in other
    rounds of the persistent grid and next to other neighbours each time; payloads, scales and
    outputs must be the same bytes (the random streams are keyed by seed, worker and global
    coordinate, no result passes through an atomic, and every chunk is reduced in one fixed
    order)."""
    l, bits, W = 14, 4, 8
    n = (37 << l) + 4321
    xs = [_rand(n, torch.bfloat16, 4000 + w, scale=10.0 ** (-1 - (w % 3))) for w in range(W)]
    nb = thc.thc_payload_bytes(n, l, bits)
    P = thc.thc_num_chunks(n, l)
    seen = None
    for lead in (0, 1, 7, 100):
        lead_n = lead << l
        first = dict(grads=[_rand(lead_n, torch.bfloat16, 77 + w) for w in range(W)] if lead else
                     [torch.empty(0, dtype=torch.bfloat16, device=DEV) for _ in range(W)],
                     n=lead_n, seed=9,
                     payloads=[torch.empty(thc.thc_payload_bytes(lead_n, l, bits), dtype=torch.uint8, device=DEV)
                               for _ in range(W)],
                     scale=torch.empty(max(lead, 1), device=DEV), out=torch.empty(max(lead_n, 1), device=DEV))
        mine = dict(grads=xs, n=n, seed=1234,
                    payloads=[torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)],
                    scale=torch.full((P,), -1.0, device=DEV), out=torch.full((n,), float("nan"), device=DEV))
        batch = [first, mine]
        ws = torch.empty(thc.thc_batch_workspace_bytes([lead_n, n], W, l), dtype=torch.uint8, device=DEV)
        print(f"determinism: bucket of {P} chunks after {lead} chunks", flush=True)
        thc.thc_encode_all_batch(batch, l, bits, ws)
        thc.thc_aggregate_decode_batch(batch, l, bits, ws)
        torch.cuda.synchronize()
        assert not thc.thc_encode_all_timed_out(ws)
        got = (torch.cat(mine["payloads"]).clone(), mine["scale"].clone(), mine["out"].clone())
        if seen is None:
            seen = got
        else:
            assert all(torch.equal(a, b) for a, b in zip(seen, got)), f"results moved with {lead} leading chunks"
