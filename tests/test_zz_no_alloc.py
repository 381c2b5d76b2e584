"""thc_encode_all_static (the entry point that allocates nothing: its workspace is a fixed
device array inside the library) against thc_encode_all, through the C ABI: identical
scales and payload bytes on two calls in a row, the second with a smaller input, and on
the shapes that take the unfused fallback; sizes beyond the array are refused."""
import pytest
import torch

import paper_2407_01378_amd as thc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn(n, generator=g, device=DEV) * scale).to(dtype)


def _both(xs, l, seed, bits):
    W, n = len(xs), xs[0].numel()
    P = thc.thc_num_chunks(n, l)
    nb = thc.thc_payload_bytes(n, l, bits)
    got = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    ref = [torch.full((nb,), 0x55, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sc_got = torch.full((P,), -1.0, device=DEV)
    sc_ref = torch.full((P,), -2.0, device=DEV)
    flag = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    ws = torch.full((thc.thc_encode_all_workspace_bytes(W, n, l),), 0xFF, dtype=torch.uint8, device=DEV)
    thc.thc_encode_all_static(xs, l, seed, bits, got, sc_got, flag)
    thc.thc_encode_all(xs, l, seed, bits, ref, sc_ref, ws)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0, "a bounded wait expired"
    assert not thc.thc_encode_all_timed_out(ws)
    assert torch.equal(sc_got, sc_ref), "scales differ"
    for w in range(W):
        assert torch.equal(got[w], ref[w]), f"payload of worker {w} differs"


@pytest.mark.parametrize("l,bits,W,dtype", [(14, 4, 8, torch.bfloat16), (14, 8, 3, torch.float32),
                                            (10, 4, 4, torch.float32)])
def test_static_workspace_form_matches_on_two_calls_in_a_row(l, bits, W, dtype):
    c = 1 << l
    for k, n in enumerate((41 * c + 77, 5 * c + 3)):   # the second call is smaller
        print(f"static l={l} bits={bits} W={W} dtype={dtype} n={n}", flush=True)
        xs = [_rand(n, dtype, 1000 + 10 * k + w, scale=10.0 ** (-1 - (w % 3))) for w in range(W)]
        _both(xs, l, 50 + k, bits)


def test_sizes_beyond_the_array_are_refused_and_null_flag_is_allowed():
    l, bits, W = 14, 4, 8
    n_ok = 3 << l
    xs = [_rand(n_ok, torch.bfloat16, 5 + w) for w in range(W)]
    pay = [torch.empty(thc.thc_payload_bytes(n_ok, l, bits), dtype=torch.uint8, device=DEV) for _ in range(W)]
    sc = torch.empty(thc.thc_num_chunks(n_ok, l), device=DEV)
    thc.thc_encode_all_static(xs, l, 1, bits, pay, sc, None)
    torch.cuda.synchronize()
    # the largest size whose workspace still fits, plus one chunk
    chunks = 1
    while thc.thc_encode_all_workspace_bytes(W, (chunks + 1) << l, l) <= thc.THC_STATIC_SCRATCH_BYTES:
        chunks += 1
    n_big = (chunks + 1) << l
    big = [torch.zeros(n_big, dtype=torch.bfloat16, device=DEV)] * W
    pay_big = [torch.empty(thc.thc_payload_bytes(n_big, l, bits), dtype=torch.uint8, device=DEV)] * W
    with pytest.raises(thc.ThcError) as e:
        thc.thc_encode_all_static(big, l, 1, bits, pay_big, torch.empty(chunks + 1, device=DEV), None)
    assert e.value.status == -6
