"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element on the same seeded inputs.  Bars: rotation, scales, payload bytes and
integer sums bit-exact; decoded output within 1e-5 relative L2 of the float64
definition fed the same sums and scales."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from synth import generate, to_numpy_bits, workload

from gpu_util import DEV, check_against_oracle, run_path, sums_to_numpy

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3, heavy=True):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    if heavy:
        x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available()
    thc.lib()


# ---------------------------------------------------------------- rotation alone
@pytest.mark.parametrize("l", [1, 2, 3, 4, 5, 7, 10, 13, 14])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rht_forward_and_inverse_bit_exact(l, dtype):
    c = 1 << l
    n = 3 * (1 << 14) + 5 * c + (c // 2 + 1 if c > 2 else 1)        # several tiles, ragged tail
    print(f"rht l={l} dtype={dtype} n={n}", flush=True)
    x = _rand(n, dtype, 100 + l)
    P = thc.thc_num_chunks(n, l)
    y = torch.full((P * c,), float("nan"), device=DEV)
    thc.rht_forward(x, l, 41, y)
    back = torch.full((n,), float("nan"), device=DEV)
    thc.rht_inverse(y, n, l, 41, back)
    torch.cuda.synchronize()
    hx = to_numpy_bits(x)
    bf = dtype == torch.bfloat16
    y32 = O.rht_forward(hx, l, 41, dtype=np.float32, bf16=bf)
    assert (y.cpu().numpy() == y32).all()
    y64 = O.rht_forward(hx, l, 41, dtype=np.float64, bf16=bf)
    assert np.linalg.norm(y.cpu().numpy() - y64) <= 1e-6 * np.linalg.norm(y64)
    assert (back.cpu().numpy() == O.rht_inverse(y32, n, l, 41, dtype=np.float32)).all()
    xf = x.float().cpu().numpy()
    assert np.linalg.norm(back.cpu().numpy() - xf) <= 1e-6 * np.linalg.norm(xf)


# ------------------------------------------------------------------ whole path
@pytest.mark.parametrize("l,bits,W,dtype", [
    (14, 4, 8, torch.bfloat16), (14, 2, 8, torch.bfloat16), (14, 8, 8, torch.bfloat16),
    (14, 4, 8, torch.float32), (10, 4, 4, torch.float32), (10, 8, 3, torch.bfloat16),
    (12, 2, 5, torch.float32), (6, 4, 2, torch.float32), (3, 8, 2, torch.bfloat16),
    (1, 2, 3, torch.float32), (2, 4, 17, torch.float32), (14, 4, 18, torch.bfloat16),
    (11, 4, 33, torch.float32), (14, 8, 20, torch.float32),
])
def test_whole_path_matches_oracle(l, bits, W, dtype):
    c = 1 << l
    n = 2 * (1 << 14) + 3 * c + (c // 2 + 1 if c > 2 else 1)
    print(f"path l={l} bits={bits} W={W} dtype={dtype} n={n}", flush=True)
    xs = [_rand(n, dtype, 1000 * l + w, scale=10.0 ** (-1 - (w % 4))) for w in range(W)]
    got = run_path(xs, l, 9, bits)
    check_against_oracle(xs, got, l, 9, bits)


def test_encode_with_own_scale_and_scale_out():
    l, bits, n = 14, 4, 2 * (1 << 14) + 777
    x = _rand(n, torch.bfloat16, 5)
    P = thc.thc_num_chunks(n, l)
    pay = torch.zeros(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV)
    sc = torch.full((P,), -1.0, device=DEV)
    thc.thc_encode(x, l, 3, 2, bits, None, pay, sc)
    torch.cuda.synchronize()
    hx = to_numpy_bits(x)
    y = O.rht_forward(hx, l, 3, dtype=np.float32, bf16=True)
    s = O.chunk_absmax(y, l)
    assert (sc.cpu().numpy() == s).all()
    idx = O.quantize(y, s, l, 2, 3, bits, dtype=np.float32)
    assert (pay.cpu().numpy() == O.pack(idx, bits)).all()
    # each chunk's extreme coordinate lands on an end of the grid
    a = np.abs(y).reshape(P, -1).argmax(axis=1)
    ends = idx.reshape(P, -1)[np.arange(P), a]
    assert set(ends.tolist()) <= {0, 15}


# ------------------------------------------------------------------- edge cases
def test_empty_input_is_a_no_op():
    e32 = torch.empty(0, device=DEV)
    e8 = torch.empty(0, dtype=torch.uint8, device=DEV)
    thc.rht_forward(e32, 10, 0, e32)
    thc.rht_inverse(e32, 0, 10, 0, e32)
    thc.thc_chunk_absmax(e32, 10, 0, e32)
    thc.thc_encode(e32, 10, 0, 0, 4, None, e8)
    thc.thc_aggregate([e8], 0, 10, 4, e8)
    thc.thc_decode(e8, e32, 1, 0, 10, 0, 4, e32)
    torch.cuda.synchronize()


@pytest.mark.parametrize("n", [1, 2, (1 << 14) - 1, 1 << 14, (1 << 14) + 1])
def test_tiny_and_boundary_sizes(n):
    print(f"boundary n={n}", flush=True)
    xs = [_rand(n, torch.float32, 7 + w, heavy=False) for w in range(2)]
    got = run_path(xs, 14, 1, 4)
    check_against_oracle(xs, got, 14, 1, 4)


def test_all_zero_and_partly_zero_chunks():
    l, c, bits = 14, 1 << 14, 4
    n = 4 * c
    xs = [_rand(n, torch.bfloat16, 20 + w) for w in range(3)]
    for x in xs:
        x[:c] = 0                       # chunk 0 zero for every worker
    xs[0][c:2 * c] = 0                  # chunk 1 zero for worker 0 only
    xs[1][2 * c + 5:3 * c] = 0          # chunk 2 of worker 1: a handful of non-zeros
    got = run_path(xs, l, 2, bits)
    check_against_oracle(xs, got, l, 2, bits)
    assert got["scale"][0].item() == 0
    assert (got["payloads"][0][: c // 2] == 0).all()
    assert (got["out"][:c] == 0).all()
    assert torch.isfinite(got["out"]).all()


@pytest.mark.parametrize("l,bits,dtype", [(14, 4, torch.float32), (14, 8, torch.bfloat16), (10, 4, torch.bfloat16),
                                          (10, 8, torch.float32), (3, 2, torch.float32), (12, 2, torch.bfloat16)])
def test_scales_too_small_for_the_reciprocal_step(l, bits, dtype):
    """Chunks whose scale is below and around 2^-120, where L / (2 s) is not finite in fp32:
    sent like all-zero chunks (tuned chunk-2^14 kernels and the kernels for every other chunk
    size), against the oracle."""
    c = 1 << l
    n = 6 * c - 1
    xs = []
    for w in range(3):
        x = _rand(n, torch.float32, 40 + w, scale=1.0)
        x[:c] *= 2.0 ** -131
        x[c:2 * c] *= 2.0 ** -123
        x[2 * c:3 * c] *= 2.0 ** -121
        x[3 * c:4 * c] *= 2.0 ** -118
        xs.append(x.to(dtype))
    print(f"tiny scales l={l} bits={bits} dtype={dtype}", flush=True)
    got = run_path(xs, l, 4, bits)
    check_against_oracle(xs, got, l, 4, bits)
    assert 0 < got["scale"][0].item() < 2.0 ** -121
    assert (got["payloads"][0][: c * bits // 8] == 0).all()


def test_payload_and_sums_do_not_write_past_their_end():
    l, bits, W = 10, 4, 3
    n = 5 * 1024 + 100
    nb = thc.thc_payload_bytes(n, l, bits)
    P = thc.thc_num_chunks(n, l)
    xs = [_rand(n, torch.float32, 50 + w) for w in range(W)]
    guard = 64
    pays = [torch.full((nb + guard,), 0x5A, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sums = torch.full(((P << l) + guard,), 0x5A, dtype=torch.uint8, device=DEV)
    out = torch.full((n + guard,), 123.0, device=DEV)
    sc = torch.empty(P, device=DEV)
    am = torch.empty(W * P, device=DEV)
    for w in range(W):
        thc.thc_chunk_absmax(xs[w], l, 4, am[w * P:(w + 1) * P])
    thc.thc_scale_reduce(am, W, P, sc)
    for w in range(W):
        thc.thc_encode(xs[w], l, 4, w, bits, sc, pays[w][:nb])
    thc.thc_aggregate([p[:nb] for p in pays], n, l, bits, sums[: P << l])
    thc.thc_decode(sums[: P << l], sc, W, n, l, 4, bits, out[:n])
    torch.cuda.synchronize()
    for p in pays:
        assert (p[nb:] == 0x5A).all()
    assert (sums[P << l:] == 0x5A).all()
    assert (out[n:] == 123.0).all()


def test_aggregate_is_exact_on_extreme_payloads():
    """All-ones payloads from the maximum number of workers a byte can hold."""
    l, n = 10, 4096
    for bits, W in [(4, 17), (2, 85), (8, 1), (8, 257), (4, 40)]:
        nb = thc.thc_payload_bytes(n, l, bits)
        pays = [torch.full((nb,), 0xFF, dtype=torch.uint8, device=DEV) for _ in range(W)]
        sb = thc.thc_sum_bytes(W, bits)
        sums = torch.zeros(n, dtype=torch.uint8 if sb == 1 else torch.int16, device=DEV)
        thc.thc_aggregate(pays, n, l, bits, sums)
        torch.cuda.synchronize()
        assert (sums_to_numpy(sums) == W * ((1 << bits) - 1)).all(), (bits, W)


# ------------------------------------------------ workloads, bench launch configuration
def test_tiny_workload_in_full():
    wl = workload("tiny")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path(xs, wl.chunk_log2, 0, 4)
    check_against_oracle(xs, got, wl.chunk_log2, 0, 4)


def _sample_chunks(P, k, seed):
    rng = np.random.default_rng(seed)
    pick = {0, P - 1, P // 2}
    pick |= set(rng.integers(0, P, size=k).tolist())
    return sorted(pick)


def _protocol_chunks(wl, n, seed, k=256):
    """First and last (padded) chunk, the chunks on both sides of every segment boundary
    below n, and k random ones: chunks are independent, so this samples the whole."""
    P = O.num_chunks(n, 14)
    pick = set(_sample_chunks(P, k, seed))
    for e in np.cumsum([sg.size for sg in wl.segments]):
        if 0 < e < n:
            pick |= {int(e - 1) >> 14, int(e) >> 14}
    return sorted(p for p in pick if p < P)


@pytest.mark.parametrize("quarter", [0, 1, 2, 3])
def test_resnet50_sized_in_full(quarter):
    """Every one of the 1,560 chunks, a quarter per test case."""
    wl = workload("resnet50")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path(xs, 14, 0, 4)
    P = O.num_chunks(wl.n, 14)
    chunks = list(range(quarter * P // 4, (quarter + 1) * P // 4))
    print(f"resnet50 chunks {chunks[0]}..{chunks[-1]} of {P}", flush=True)
    check_against_oracle(xs, got, 14, 0, 4, chunks=chunks)


def test_bert_base_sized_sampled_chunks_with_sparse_embedding():
    wl = workload("bert_base")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path(xs, 14, 0, 4)
    emb = wl.segments[0].size // (1 << 14)
    chunks = sorted(set(_protocol_chunks(wl, wl.n, 2)) | set(range(0, emb, emb // 12)) | {emb, emb + 1})
    print(f"bert_base {len(chunks)} chunks", flush=True)
    check_against_oracle(xs, got, 14, 0, 4, chunks=chunks)
    assert (got["scale"][:emb] == 0).any()          # all-zero chunks exist and were exercised


@pytest.mark.parametrize("bits", [2, 8])
def test_gpt_345m_sampled_chunks(bits):
    wl = workload("gpt_345m")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path(xs, 14, 0, bits)
    chunks = _protocol_chunks(wl, wl.n, bits)
    print(f"gpt_345m bits={bits} {len(chunks)} chunks of {O.num_chunks(wl.n, 14)}", flush=True)
    check_against_oracle(xs, got, 14, 0, bits, chunks=chunks)


def test_gpt_1p3b_buckets_sampled_chunks():
    """One full bucket (25 * 2^20 coordinates, 1600 chunks) and the ragged last
    bucket (15,494,400 coordinates, 946 chunks), W = 8, 4 bits: the launch shapes
    the benchmark times."""
    wl = workload("gpt_1p3b")
    full, last = wl.buckets()[0][1], wl.buckets()[-1][1]
    for k, n in enumerate((full, last)):
        xs = [generate(wl, w, DEV, max_elems=n) for w in range(wl.W)]
        got = run_path(xs, 14, 7 + k, 4)
        chunks = _protocol_chunks(wl, n, k)
        print(f"gpt_1p3b bucket of {n}: {len(chunks)} chunks", flush=True)
        check_against_oracle(xs, got, 14, 7 + k, 4, chunks=chunks)
        del xs, got


def test_coordinates_beyond_2_to_32():
    """4 Gi + 3 chunks + 100 coordinates per worker: global indices (Philox counters, byte
    offsets, chunk numbers) cross 2^32.  Both forms, chunks sampled on both sides of the
    boundary and at the ragged end."""
    from gpu_util import check_chunks_sliced, run_path_fused
    l, bits, W = 14, 4, 2
    n = (1 << 32) + 3 * (1 << 14) + 100
    print(f"large n={n}", flush=True)
    g = torch.Generator(device=DEV)
    g.manual_seed(4)
    block = (torch.randn(1 << 24, generator=g, device=DEV) * 1e-3).to(torch.bfloat16)
    xs = []
    for w in range(W):
        x = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        full = n // block.numel()
        x[:full * block.numel()].view(full, -1).copy_(block.roll(1000 * w + 1).unsqueeze(0).expand(full, -1))
        x[full * block.numel():] = block[:n - full * block.numel()] * (w + 1)
        xs.append(x)
    P = O.num_chunks(n, l)
    edge = (1 << 32) >> l
    chunks = [0, 1, edge - 2, edge - 1, edge, edge + 1, P - 2, P - 1, P // 3]
    got = run_path_fused(xs, l, 3, bits, keep_sums=False)
    check_chunks_sliced(xs, got, l, 3, bits, chunks)
    fused_out = got["out"]
    fused_pay = got["payloads"]
    print("large n: one-call-per-step form", flush=True)
    got = run_path(xs, l, 3, bits)
    check_chunks_sliced(xs, got, l, 3, bits, chunks)
    # the two forms agree everywhere, not only on the sampled chunks
    for a, b in zip(fused_pay, got["payloads"]):
        assert torch.equal(a, b)
    assert torch.equal(fused_out, got["out"])


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("n", [9, 10, 1, 101])
def test_chunks_of_two_coordinates_and_a_partial_last_payload_byte(n, bits):
    """The smallest chunk: with 2-bit indices an odd number of chunks ends inside a payload
    byte (thc_payload_bytes rounds up); both forms against the oracle."""
    from gpu_util import run_path_fused
    xs = [_rand(n, torch.float32, 60 + w, heavy=False) for w in range(3)]
    print(f"chunk 2, n={n} bits={bits}", flush=True)
    assert thc.thc_payload_bytes(n, 1, bits) == (((n + 1) // 2) * 2 * bits + 7) // 8
    check_against_oracle(xs, run_path(xs, 1, 8, bits), 1, 8, bits)
    check_against_oracle(xs, run_path_fused(xs, 1, 8, bits), 1, 8, bits)
