"""TopKC on the GPU against its oracle: per-worker norms, summed norms, selected indices,
fp16 chunk sums and the dense estimate, all bit-exact."""
import numpy as np
import pytest
import torch

import paper_2407_01378_amd as thc
from oracle import topkc as K
from synth import generate, to_numpy_bits, workload

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _data(n, dtype, W, seed, clustered=True):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    xs = []
    seg = 1000
    scale = 10.0 ** (torch.rand((n + seg - 1) // seg, generator=g, device=DEV) * 3 - 4)
    scale = scale.repeat_interleave(seg)[:n] if clustered else torch.full((n,), 1e-2, device=DEV)
    for w in range(W):
        xs.append((torch.randn(n, generator=g, device=DEV) * scale).to(dtype))
    return xs


def run_topkc(xs, C, J):
    W, n = len(xs), xs[0].numel()
    P = thc.topkc_num_chunks(n, C)
    norms_all = torch.full((W * P,), float("nan"), dtype=torch.float16, device=DEV)
    s = torch.full((P,), float("nan"), dtype=torch.float16, device=DEV)
    idx = torch.full((J,), -1, dtype=torch.int32, device=DEV)
    ws = torch.full((thc.topkc_select_workspace_bytes(P),), 0xFF, dtype=torch.uint8, device=DEV)
    vals = torch.full((J * C,), float("nan"), dtype=torch.float16, device=DEV)
    out = torch.full((n,), float("nan"), device=DEV)
    for w in range(W):
        thc.topkc_chunk_norms(xs[w], C, norms_all[w * P:(w + 1) * P])
    thc.topkc_sum_norms(norms_all, W, P, s)
    thc.topkc_select(s, J, idx, ws)
    thc.topkc_gather_sum(xs, C, idx, J, vals)
    thc.topkc_scatter_mean(vals, idx, J, C, W, out)
    torch.cuda.synchronize()
    return dict(norms=norms_all.view(W, P), s=s, indices=idx, values=vals.view(J, C), out=out)


def _bits16(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check(xs, got, C, J):
    bf16 = xs[0].dtype == torch.bfloat16
    ref = K.pipeline([to_numpy_bits(x) for x in xs], C, J, bf16=bf16)
    for w in range(len(xs)):
        assert (_bits16(got["norms"][w]) == ref["norms"][w].view(np.uint16)).all(), f"norms of worker {w}"
    assert (_bits16(got["s"]) == ref["s"].view(np.uint16)).all(), "summed norms"
    assert (got["indices"].cpu().numpy().view(np.uint32) == ref["indices"]).all(), "selected indices"
    assert (_bits16(got["values"]) == ref["values"].view(np.uint16)).all(), "chunk sums"
    assert (got["out"].cpu().numpy() == ref["out"]).all(), "dense estimate"
    return ref


@pytest.mark.parametrize("n,C,J,W,dtype", [
    (100_000, 64, 100, 4, torch.float32), (100_003, 128, 37, 8, torch.bfloat16),
    (1 << 20, 64, 1, 3, torch.bfloat16), (1 << 20, 64, 16384, 3, torch.float32),     # J = 1 and J = P
    (999_999, 8, 5000, 2, torch.float32), (300_000, 512, 100, 5, torch.bfloat16),
    (70, 64, 2, 2, torch.float32), (5_000_000, 128, 3000, 8, torch.bfloat16),
])
def test_topkc_matches_oracle(n, C, J, W, dtype):
    print(f"topkc n={n} C={C} J={J} W={W} dtype={dtype}", flush=True)
    xs = _data(n, dtype, W, seed=n % 1000 + C)
    check(xs, run_topkc(xs, C, J), C, J)


@pytest.mark.parametrize("offset", [0, 1, 2, 3])
@pytest.mark.parametrize("n", [1, 2, 3, 5, 64, 1000, 65_537, 1_000_003])
def test_scatter_fills_unaligned_outputs_exactly(offset, n):
    """The zero fill under topkc_scatter_mean writes 16 bytes at a time in the aligned
    middle of the output and word by word at its ends: nothing outside [0, n) may change
    and nothing inside may be left over, wherever the output starts."""
    C, W = 8, 2
    J = min(3, (n + C - 1) // C)
    buf = torch.full((n + 8,), 7.0, device=DEV)
    out = buf[offset:offset + n]
    vals = torch.full((J * C,), 4.0, dtype=torch.float16, device=DEV)
    idx = torch.arange(J, dtype=torch.int32, device=DEV)
    thc.topkc_scatter_mean(vals, idx, J, C, W, out)
    torch.cuda.synchronize()
    want = torch.zeros(n, device=DEV)
    want[:min(n, J * C)] = 2.0
    assert torch.equal(out, want)
    assert (buf[:offset] == 7.0).all() and (buf[offset + n:] == 7.0).all()


def test_topkc_many_ties_and_zero_chunks():
    """Most chunks are exactly zero (their fp16 norms tie at 0) and many non-zero chunks tie
    too: the J-th place falls among equal keys and must go to the lowest indices."""
    n, C, W = 1 << 18, 64, 3
    P = n // C
    xs = [torch.zeros(n, device=DEV) for _ in range(W)]
    for w in range(W):
        for p in range(0, P, 5):
            xs[w][p * C] = 1.0 + (p % 3)          # three distinct non-zero norm values, repeated
    for J in (1, 7, P // 5, P // 5 + 10, P):
        got = run_topkc(xs, C, J)
        ref = check(xs, got, C, J)
        assert len(set(ref["indices"].tolist())) == J


def test_topkc_underflowing_norms_are_kept_as_fp16_gives_them():
    """Gradients of size 1e-5: squared chunk norms around 6e-9 are below fp16's smallest
    subnormal and round to zero, as the paper's half-precision norms do."""
    n, C, W, J = 1 << 16, 64, 2, 10
    xs = [torch.full((n,), 1e-5, device=DEV) for _ in range(W)]
    xs[0][4096:4096 + 64] = 0.5
    got = run_topkc(xs, C, J)
    ref = check(xs, got, C, J)
    assert ref["indices"][0] == 0 or 64 in ref["indices"]      # the one large chunk is chunk 64
    assert 64 in ref["indices"].tolist()
    assert (ref["s"].astype(np.float32) == 0).sum() == n // C - 1


def test_topkc_argument_checks():
    x = torch.zeros(1000, device=DEV)
    norms = torch.zeros(100, dtype=torch.float16, device=DEV)
    with pytest.raises(thc.ThcError):
        thc.topkc_chunk_norms(x, 48, norms)        # C not a power of two
    with pytest.raises(thc.ThcError):
        thc.topkc_chunk_norms(x, 1024, norms)      # C too large
    s = torch.zeros(16, dtype=torch.float16, device=DEV)
    idx = torch.zeros(32, dtype=torch.int32, device=DEV)
    ws = torch.zeros(thc.topkc_select_workspace_bytes(16), dtype=torch.uint8, device=DEV)
    with pytest.raises(thc.ThcError):
        thc.topkc_select(s, 17, idx, ws)           # J > P
    with pytest.raises(thc.ThcError):
        thc.topkc_select(s, 0, idx, ws)
    with pytest.raises(thc.ThcError):
        thc.topkc_select(s, 4, idx, ws[:8])        # workspace too small


def test_topkc_on_headline_workload_slice():
    """50 M coordinates of the 1.3B workload's gradients (bf16, W = 8), C = 64, J chosen for
    about 2 bits per coordinate: every stage compared with the oracle."""
    wl = workload("gpt_1p3b")
    n, C = 50_000_000, 64
    J = int(0.11 * n / C)
    xs = [generate(wl, w, torch.device(DEV), max_elems=n) for w in range(wl.W)]
    got = run_topkc(xs, C, J)
    check(xs, got, C, J)
    print(f"bits per coordinate: {K.bits_per_coordinate(J, C, n):.3f}", flush=True)


def test_topkc_offsets_beyond_2_to_32():
    """More than 2^32 coordinates, all zero except five chunks on both sides of the 2^32
    boundary and at the ragged end: chunk numbers, gather and scatter offsets cross 32
    bits.  The oracle runs on the five chunks laid side by side, which is the same problem
    (zero chunks have norm 0 and cannot be selected ahead of them)."""
    C, W, J = 64, 2, 5
    n = (1 << 32) + 64 * 10 + 17
    P = thc.topkc_num_chunks(n, C)
    edge = (1 << 32) // C
    picks = [7, edge - 1, edge + 3, P - 5, P - 1]
    print(f"topkc large n={n} P={P} picks={picks}", flush=True)
    g = torch.Generator(device=DEV)
    g.manual_seed(12)
    xs = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for _ in range(W)]
    compact = [np.zeros(J * C, dtype=np.uint16) for _ in range(W)]
    for w in range(W):
        for k, p in enumerate(picks):
            ln = min(n, (p + 1) * C) - p * C
            v = (torch.randn(ln, generator=g, device=DEV) * (0.05 * (k + 1))).to(torch.bfloat16)
            xs[w][p * C:p * C + ln] = v
            compact[w][k * C:k * C + ln] = to_numpy_bits(v)
    got = run_topkc(xs, C, J)
    ref = K.pipeline(compact, C, J, bf16=True)
    assert ref["indices"].tolist() == list(range(J))
    assert got["indices"].cpu().numpy().tolist() == picks
    sel = torch.tensor(picks, device=DEV)
    for w in range(W):
        assert (_bits16(got["norms"][w][sel]) == ref["norms"][w].view(np.uint16)).all()
        assert int(got["norms"][w].count_nonzero()) == J
    assert (_bits16(got["s"][sel]) == ref["s"].view(np.uint16)).all()
    assert int(got["s"].count_nonzero()) == J
    assert (_bits16(got["values"]) == ref["values"].view(np.uint16)).all()
    nonzero = 0
    for k, p in enumerate(picks):
        ln = min(n, (p + 1) * C) - p * C
        seg = got["out"][p * C:p * C + ln].cpu().numpy()
        assert (seg == ref["out"][k * C:k * C + ln]).all(), f"estimate differs in chunk {p}"
        nonzero += int(np.count_nonzero(seg))
    assert int(got["out"].count_nonzero()) == nonzero


def _sampled_check(xs, C, J):
    """Every stage of a TopKC round on inputs too large for the oracle to run whole: norms,
    summed norms, chunk sums and the estimate against the oracle on sampled chunks (the
    first and last ones, both sides of every 2^22-chunk boundary, 2000 random); the
    selection by the properties that define it."""
    W, n = len(xs), xs[0].numel()
    bf16 = xs[0].dtype == torch.bfloat16
    P = thc.topkc_num_chunks(n, C)
    got = run_topkc(xs, C, J)
    rng = np.random.default_rng(5)
    picks = {0, 1, P - 2, P - 1}
    for b in range(1 << 22, P, 1 << 22):
        picks.update((b - 1, b))
    picks.update(int(p) for p in rng.integers(0, P, 2000))
    picks = np.array(sorted(picks), dtype=np.int64)

    def chunks_of(x, which):   # the given chunks of one gradient, side by side, zero-padded, as raw bits
        pos = (torch.as_tensor(which, device=DEV)[:, None] * C + torch.arange(C, device=DEV)[None, :]).reshape(-1)
        v = x[pos.clamp_max(n - 1)]
        v[pos >= n] = 0
        return to_numpy_bits(v)

    sel = torch.as_tensor(picks, device=DEV)
    ref_norms = [K.chunk_norms(chunks_of(x, picks), C, bf16=bf16) for x in xs]
    for w in range(W):
        assert (_bits16(got["norms"][w][sel]) == ref_norms[w].view(np.uint16)).all(), f"norms of worker {w}"
    assert (_bits16(got["s"][sel]) == K.sum_fp16(ref_norms).view(np.uint16)).all(), "summed norms"
    # selection: J distinct chunks, ascending; nothing left out is larger than anything taken,
    # and among equals of the smallest taken value the lowest chunk numbers are taken
    idx = got["indices"].to(torch.int64)
    assert int(idx.min()) >= 0 and int(idx.max()) < P and bool((idx[1:] > idx[:-1]).all())
    s = got["s"].float()
    taken = torch.zeros(P, dtype=torch.bool, device=DEV)
    taken[idx] = True
    thr = float(s[taken].min())
    assert float(s[~taken].max()) <= thr
    eq_taken = taken[torch.nonzero(s == thr).flatten()]
    k = int(eq_taken.sum())
    assert bool(eq_taken[:k].all()) and not bool(eq_taken[k:].any()), "ties: lowest chunk numbers first"
    # chunk sums and estimate on sampled selected chunks, zeros on sampled chunks left out
    js = np.unique(np.concatenate([[0, 1, J - 2, J - 1], rng.integers(0, J, 1500)])).astype(np.int64)
    chosen = idx[torch.as_tensor(js, device=DEV)].cpu().numpy()
    ref_vals = K.gather_sum([chunks_of(x, chosen) for x in xs], C, np.arange(len(chosen)), bf16=bf16)
    assert (_bits16(got["values"][torch.as_tensor(js, device=DEV)]) == ref_vals.view(np.uint16)).all(), "chunk sums"
    ref_out = K.scatter_mean(ref_vals, np.arange(len(chosen)), C, W, len(chosen) * C)
    out_pos = torch.as_tensor(chosen, device=DEV)[:, None] * C + torch.arange(C, device=DEV)[None, :]
    inside = (out_pos < n).cpu().numpy().reshape(-1)
    assert (got["out"][out_pos.clamp_max(n - 1)].cpu().numpy().reshape(-1)[inside] == ref_out[inside]).all(), "estimate"
    left_out = torch.as_tensor(picks[~taken[sel].cpu().numpy()], device=DEV)
    gone = (left_out[:, None] * C + torch.arange(C, device=DEV)[None, :]).reshape(-1)
    assert int(got["out"][gone[gone < n]].count_nonzero()) == 0
    assert int(got["out"].count_nonzero()) == int(got["values"].count_nonzero())


def test_topkc_full_size_sampled_against_the_oracle():
    """The whole 1.3 B-coordinate gradients of the headline workload (bf16, W = 8, C = 64, J
    for 2 bits per coordinate), the shapes and launch configurations `bench.py --topkc`
    times: the norm kernel's grid-stride loop and the gather / scatter grids beyond 2^24
    threads only run at this size."""
    wl = workload("gpt_1p3b")
    n, C = wl.n, 64
    J = max(1, int((2.0 / 16.0 - 1.0 / C) * n / C))
    print(f"topkc full size n={n} J={J}", flush=True)
    _sampled_check([generate(wl, w, torch.device(DEV)) for w in range(wl.W)], C, J)


def test_topkc_large_fp32_sampled_against_the_oracle():
    """fp32 input long enough for the norm kernel's grid-stride loop (more than 2^25 groups
    of 8), with a ragged last group and chunk."""
    n, C, J, W = (300 << 20) + 13, 128, 50_000, 2
    print(f"topkc large fp32 n={n} J={J}", flush=True)
    _sampled_check(_data(n, torch.float32, W, seed=77), C, J)


@pytest.mark.parametrize("offset", [0, 1, 3, 8])
@pytest.mark.parametrize("P,J", [(5, 2), (1000, 1000), (70_001, 333), (70_008, 69_000)])
def test_topkc_select_on_unaligned_and_ragged_key_arrays(offset, P, J):
    """The selection reads its keys 8 at a time when the array is 16-byte aligned and one at
    a time otherwise; both against the oracle, with many equal keys and zeros in runs."""
    g = torch.Generator(device=DEV)
    g.manual_seed(P + offset)
    vals = (torch.randint(0, 40, (P + offset,), generator=g, device=DEV).float() / 8.0)
    vals[offset + P // 3: offset + P // 2] = 0.0
    s = vals.half()[offset:]
    assert s.data_ptr() % 16 == (2 * offset) % 16
    idx = torch.full((J,), -1, dtype=torch.int32, device=DEV)
    ws = torch.full((thc.topkc_select_workspace_bytes(P),), 0xFF, dtype=torch.uint8, device=DEV)
    print(f"topkc select offset={offset} P={P} J={J}", flush=True)
    thc.topkc_select(s, J, idx, ws)
    torch.cuda.synchronize()
    ref = K.select(s.cpu().numpy(), J)
    assert (idx.cpu().numpy().view(np.uint32) == ref).all()
