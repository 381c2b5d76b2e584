"""Helpers for the GPU parity tests: run the path through the C ABI binding."""
import numpy as np
import torch

import paper_2407_01378_amd as thc
from oracle import thc as O
from synth import to_numpy_bits

DEV = "cuda:0"


def run_path_fused(xs, l, seed, bits, keep_sums=True):
    """thc_encode_all -> thc_aggregate_decode on the GPU; same result keys as run_path
    (absmax is not produced by the fused form)."""
    W = len(xs)
    n = xs[0].numel()
    dev = xs[0].device
    P = thc.thc_num_chunks(n, l)
    scale = torch.full((P,), -1.0, dtype=torch.float32, device=dev)
    nb = thc.thc_payload_bytes(n, l, bits)
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=dev) for _ in range(W)]
    ws = torch.full((thc.thc_encode_all_workspace_bytes(W, n, l),), 0xFF, dtype=torch.uint8, device=dev)
    sb = thc.thc_sum_bytes(W, bits)
    sums = torch.full((P << l,), 77, dtype=torch.uint8 if sb == 1 else torch.int16, device=dev)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    thc.thc_encode_all(xs, l, seed, bits, payloads, scale, ws)
    thc.thc_aggregate_decode(payloads, scale, n, l, seed, bits, sums if keep_sums else None, out)
    torch.cuda.synchronize()
    assert not thc.thc_encode_all_timed_out(ws), "a wait inside thc_encode_all expired"
    return dict(scale=scale, payloads=payloads, sums=sums if keep_sums else None, out=out)


def run_path_timed(xs, l, seed, bits, reuse=None):
    """The form bench.py times: a workspace cleared ONCE (thc_workspace_clear), then
    thc_encode_all_cleared + thc_aggregate_decode with sums = NULL.  `reuse` is a workspace
    left by an earlier call of this function (it must have come back clear)."""
    W = len(xs)
    n = xs[0].numel()
    dev = xs[0].device
    P = thc.thc_num_chunks(n, l)
    scale = torch.full((P,), -1.0, dtype=torch.float32, device=dev)
    nb = thc.thc_payload_bytes(n, l, bits)
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=dev) for _ in range(W)]
    need = thc.thc_encode_all_workspace_bytes(W, n, l)
    if reuse is None:
        ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=dev)
        thc.thc_workspace_clear(ws)
    else:
        ws = reuse
        assert ws.numel() >= need
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    sums = None                       # the fused decoder never stores them; the fallback needs them
    if not thc.thc_aggregate_decode_is_fused(W, l, bits):
        sb = thc.thc_sum_bytes(W, bits)
        sums = torch.full((P << l,), 77, dtype=torch.uint8 if sb == 1 else torch.int16, device=dev)
    thc.thc_encode_all_cleared(xs, l, seed, bits, payloads, scale, ws)
    thc.thc_aggregate_decode(payloads, scale, n, l, seed, bits, sums, out)
    torch.cuda.synchronize()
    assert not thc.thc_encode_all_timed_out(ws), "a wait inside thc_encode_all_cleared expired"
    assert int(ws.count_nonzero()) == 0, "the workspace did not come back clear"
    return dict(scale=scale, payloads=payloads, sums=sums, out=out, workspace=ws)


def run_path(xs, l, seed, bits, own_scale=False):
    """absmax -> scale_reduce -> encode x W -> aggregate -> decode on the GPU.
    xs: list of W device tensors (fp32 or bf16).  Returns device tensors."""
    W = len(xs)
    n = xs[0].numel()
    dev = xs[0].device
    P = thc.thc_num_chunks(n, l)
    absmax = torch.full((W * P,), -1.0, dtype=torch.float32, device=dev)
    scale = torch.full((P,), -1.0, dtype=torch.float32, device=dev)
    nb = thc.thc_payload_bytes(n, l, bits)
    payloads = [torch.full((nb,), 0xAA, dtype=torch.uint8, device=dev) for _ in range(W)]
    sb = thc.thc_sum_bytes(W, bits)
    sums = torch.full((P << l,), 77, dtype=torch.uint8 if sb == 1 else torch.int16, device=dev)
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    for w in range(W):
        thc.thc_chunk_absmax(xs[w], l, seed, absmax[w * P:(w + 1) * P])
    thc.thc_scale_reduce(absmax, W, P, scale)
    for w in range(W):
        thc.thc_encode(xs[w], l, seed, w, bits, scale, payloads[w])
    thc.thc_aggregate(payloads, n, l, bits, sums)
    thc.thc_decode(sums, scale, W, n, l, seed, bits, out)
    torch.cuda.synchronize()
    return dict(absmax=absmax.view(W, P), scale=scale, payloads=payloads, sums=sums, out=out)


def sums_to_numpy(sums):
    a = sums.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def check_against_oracle(xs, got, l, seed, bits, chunks=None):
    """Element-by-element comparison with the oracle.  chunks: list of chunk
    indices to check (None = all); the oracle is run on those chunks only, with
    their global offset."""
    W = len(xs)
    n = xs[0].numel()
    c = 1 << l
    P = O.num_chunks(n, l)
    bf16 = xs[0].dtype == torch.bfloat16
    if chunks is None:
        groups = [(0, n)]
    else:
        groups = [(p * c, min(n, (p + 1) * c) - p * c) for p in sorted(set(chunks))]
    scale = got["scale"].cpu().numpy()
    absmax = got["absmax"].cpu().numpy() if "absmax" in got else None
    sums = sums_to_numpy(got["sums"]) if got.get("sums") is not None else None
    out = got["out"].cpu().numpy()
    pay = [p.cpu().numpy() for p in got["payloads"]]
    worst = 0.0
    for g0, ln in groups:
        hx = [to_numpy_bits(x[g0:g0 + ln]) for x in xs]
        ref = O.pipeline(hx, l, seed, bits, dtype=np.float32, bf16=bf16, g0=g0)
        p0, np_ = g0 // c, O.num_chunks(ln, l)
        if absmax is not None:
            assert (absmax[:, p0:p0 + np_] == ref["absmax"]).all(), f"absmax differs, chunk {p0}"
        assert (scale[p0:p0 + np_] == ref["scale"]).all(), f"scale differs, chunk {p0}"
        b0, b1 = g0 * bits // 8, ((g0 + np_ * c) * bits + 7) // 8   # (chunks of 2 x 2 bits end inside a byte)
        for w in range(W):
            same = pay[w][b0:b1] == ref["payloads"][w]
            assert same.all(), f"payload of worker {w} differs in chunk {p0}: {np.flatnonzero(~same)[:8]}"
        if sums is not None:
            assert (sums[g0:g0 + np_ * c] == ref["sums"]).all(), f"sums differ, chunk {p0}"
        # decode, stage-wise: float64 definition fed the same sums and scales
        d64 = O.decode(ref["sums"], ref["scale"].astype(np.float64), W, ln, l, seed, bits, g0=g0)
        seg = out[g0:g0 + ln]
        nrm = np.linalg.norm(d64)
        if nrm == 0:
            assert (seg == 0).all()
        else:
            err = np.linalg.norm(seg - d64) / nrm
            assert err <= 1e-5, f"decode rel-L2 {err} in chunk {p0}"
            worst = max(worst, err)
        assert (seg == ref["out"]).all(), f"decode differs from the fp32 canonical order, chunk {p0}"
    return worst


def check_chunks_sliced(xs, got, l, seed, bits, chunks):
    """check_against_oracle for arrays too large to copy to the host whole: only the
    listed chunks' slices of every array leave the device."""
    W = len(xs)
    n = xs[0].numel()
    c = 1 << l
    bf16 = xs[0].dtype == torch.bfloat16
    for p in sorted(set(chunks)):
        g0 = p * c
        ln = min(n, g0 + c) - g0
        hx = [to_numpy_bits(x[g0:g0 + ln]) for x in xs]
        ref = O.pipeline(hx, l, seed, bits, dtype=np.float32, bf16=bf16, g0=g0)
        assert float(got["scale"][p]) == float(ref["scale"][0]), f"scale differs, chunk {p}"
        if "absmax" in got:
            assert (got["absmax"][:, p].cpu().numpy() == ref["absmax"][:, 0]).all(), f"absmax differs, chunk {p}"
        b0, b1 = g0 * bits // 8, (g0 + c) * bits // 8
        for w in range(W):
            same = got["payloads"][w][b0:b1].cpu().numpy() == ref["payloads"][w]
            assert same.all(), f"payload of worker {w} differs in chunk {p}: {np.flatnonzero(~same)[:8]}"
        if got.get("sums") is not None:
            assert (sums_to_numpy(got["sums"][g0:g0 + c]) == ref["sums"]).all(), f"sums differ, chunk {p}"
        seg = got["out"][g0:g0 + ln].cpu().numpy()
        d64 = O.decode(ref["sums"], ref["scale"].astype(np.float64), W, ln, l, seed, bits, g0=g0)
        nrm = np.linalg.norm(d64)
        assert nrm == 0 or np.linalg.norm(seg - d64) / nrm <= 1e-5, f"decode rel-L2, chunk {p}"
        assert (seg == ref["out"]).all(), f"decode differs from the fp32 canonical order, chunk {p}"
