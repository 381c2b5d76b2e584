"""Parity of the launch form that bench.py times - one workspace cleared once, then
thc_encode_all_cleared and thc_aggregate_decode with sums = NULL - with the oracle,
element by element: the method's degenerate case (all-zero chunks) and every workload
configuration, the large ones on the protocol's sample of chunks (first, last, both sides
of every segment boundary, 256 random ones)."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from synth import generate, workload

from gpu_util import DEV, check_against_oracle, run_path_timed

pytestmark = pytest.mark.gpu


def _rand(n, dtype, seed, scale=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    x = x / torch.sqrt((torch.randn(3, n, generator=g, device=DEV) ** 2).mean(dim=0))
    return (x * scale).to(dtype)


def _protocol_chunks(wl, n, seed, k=256):
    P = O.num_chunks(n, 14)
    rng = np.random.default_rng(seed)
    pick = {0, P - 1, P // 2} | set(rng.integers(0, P, size=k).tolist())
    for e in np.cumsum([sg.size for sg in wl.segments]):
        if 0 < e < n:
            pick |= {int(e - 1) >> 14, int(e) >> 14}
    return sorted(p for p in pick if p < P)


@pytest.mark.parametrize("W,dtype,bits,tail", [(3, torch.bfloat16, 4, 77), (8, torch.bfloat16, 4, 78),
                                               (8, torch.float32, 4, 77), (5, torch.bfloat16, 8, 2),
                                               (8, torch.bfloat16, 2, 16383)])
def test_all_zero_and_partly_zero_chunks(W, dtype, bits, tail):
    """Chunks that are zero for every worker (scale 0: every index 0, decodes to exactly 0),
    zero for one worker only, and almost zero; twice on the same workspace.  Ragged tails
    with an odd and an even count of coordinates (bf16 takes different loaders for them)."""
    l, c = 14, 1 << 14
    n = 6 * c + tail
    ws = None
    for rep in range(2):
        xs = [_rand(n, dtype, 20 + 10 * rep + w) for w in range(W)]
        for x in xs:
            x[:c] = 0                       # chunk 0 zero for every worker
            x[4 * c:5 * c] = 0              # and chunk 4, in the middle of a workgroup's run
        xs[0][c:2 * c] = 0                  # chunk 1 zero for worker 0 only
        xs[1][2 * c + 5:3 * c] = 0          # chunk 2 of worker 1: a handful of non-zeros
        xs[W - 1][5 * c:] = 0               # the ragged last chunks zero for the last worker
        print(f"timed form, zero chunks W={W} dtype={dtype} bits={bits} rep={rep}", flush=True)
        got = run_path_timed(xs, l, 2 + rep, bits, reuse=ws)
        ws = got["workspace"]
        check_against_oracle(xs, got, l, 2 + rep, bits)
        assert got["scale"][0].item() == 0 and got["scale"][4].item() == 0
        for p in got["payloads"]:
            assert (p[: c * bits // 8] == 0).all()
        assert (got["out"][:c] == 0).all() and (got["out"][4 * c:5 * c] == 0).all()
        assert torch.isfinite(got["out"]).all()


def test_tiny_workload_in_full():
    wl = workload("tiny")                 # chunk 2^10: the cleared form's unfused fallback
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path_timed(xs, wl.chunk_log2, 0, 4)
    check_against_oracle(xs, got, wl.chunk_log2, 0, 4)


def test_resnet50_sized_sampled_quarter():
    wl = workload("resnet50")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path_timed(xs, 14, 0, 4)
    P = O.num_chunks(wl.n, 14)
    chunks = sorted(set(range(1, P, 4)) | set(_protocol_chunks(wl, wl.n, 3, k=0)))
    print(f"timed form, resnet50: {len(chunks)} of {P} chunks", flush=True)
    check_against_oracle(xs, got, 14, 0, 4, chunks=chunks)


def test_bert_base_sized_sampled_chunks_with_sparse_embedding():
    wl = workload("bert_base")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path_timed(xs, 14, 0, 4)
    emb = wl.segments[0].size // (1 << 14)
    chunks = sorted(set(_protocol_chunks(wl, wl.n, 2)) | set(range(0, emb, emb // 12)) | {emb, emb + 1})
    print(f"timed form, bert_base: {len(chunks)} chunks", flush=True)
    check_against_oracle(xs, got, 14, 0, 4, chunks=chunks)
    assert (got["scale"][:emb] == 0).any()          # all-zero chunks exist and were exercised


@pytest.mark.parametrize("bits", [2, 8])
def test_gpt_345m_sampled_chunks(bits):
    wl = workload("gpt_345m")
    xs = [generate(wl, w, DEV) for w in range(wl.W)]
    got = run_path_timed(xs, 14, 0, bits)
    chunks = _protocol_chunks(wl, wl.n, bits)
    print(f"timed form, gpt_345m bits={bits}: {len(chunks)} chunks", flush=True)
    check_against_oracle(xs, got, 14, 0, bits, chunks=chunks)


def test_gpt_1p3b_both_bucket_shapes_protocol_sample():
    """One full bucket (25 * 2^20 coordinates, 1600 chunks) and the ragged last bucket
    (15,494,400 coordinates, 946 chunks), W = 8, 4 bits, Philox seed = bucket index as in
    bench.py; both on ONE workspace, the larger first."""
    wl = workload("gpt_1p3b")
    buckets = wl.buckets()
    ws = None
    for k, n in ((0, buckets[0][1]), (len(buckets) - 1, buckets[-1][1])):
        xs = [generate(wl, w, DEV, max_elems=n) for w in range(wl.W)]
        got = run_path_timed(xs, 14, k, 4, reuse=ws)
        ws = got["workspace"]
        chunks = _protocol_chunks(wl, n, k)
        print(f"timed form, gpt_1p3b bucket {k} of {n}: {len(chunks)} chunks", flush=True)
        check_against_oracle(xs, got, 14, k, 4, chunks=chunks)
        del xs, got
