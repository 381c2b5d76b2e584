"""The one-launch forms recorded into a HIP graph: every replay must give the bytes the
eager calls give on the same inputs.  (The clearing of the workspace is a kernel, not a
memset node, and the cleared-workspace form has none at all.)  Replays alternate with
eager work and synchronisations, and each one is checked."""
import pytest
import torch

import paper_2407_01378_amd as thc

from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _rand(n, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn(n, generator=g, device=DEV) * 1e-2).to(torch.bfloat16)


@pytest.mark.parametrize("cleared", [False, True])
def test_graph_replays_match_eager_calls(cleared):
    l, bits, W = 14, 4, 8
    n = 300 * (1 << 14) + 77
    P = thc.thc_num_chunks(n, l)
    nb = thc.thc_payload_bytes(n, l, bits)
    xs = [_rand(n, 7 + w) for w in range(W)]
    pay = [torch.empty(nb, dtype=torch.uint8, device=DEV) for _ in range(W)]
    scale = torch.empty(P, device=DEV)
    out = torch.empty(n, device=DEV)
    ws = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
    thc.thc_workspace_clear(ws)
    encode = thc.thc_encode_all_cleared if cleared else thc.thc_encode_all

    def step():
        encode(xs, l, 5, bits, pay, scale, ws)
        thc.thc_aggregate_decode(pay, scale, n, l, 5, bits, None, out)

    step()                                   # warm-up outside the capture (one-time queries)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()               # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    ref_pay = [torch.empty_like(p) for p in pay]
    ref_scale, ref_out = torch.empty_like(scale), torch.empty_like(out)
    ws2 = torch.empty_like(ws)
    for rep in range(4):
        print(f"graph replay {rep} cleared={cleared}", flush=True)
        for w in range(W):                   # new inputs in the recorded buffers
            xs[w].copy_(_rand(n, 100 * rep + w))
        for p in pay:
            p.fill_(0xEE)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert not thc.thc_encode_all_timed_out(ws)
        if cleared:
            assert int(ws.count_nonzero()) == 0
        thc.thc_encode_all(xs, l, 5, bits, ref_pay, ref_scale, ws2)     # eager, between replays
        thc.thc_aggregate_decode(ref_pay, ref_scale, n, l, 5, bits, None, ref_out)
        torch.cuda.synchronize()
        assert torch.equal(scale, ref_scale)
        for a, b in zip(pay, ref_pay):
            assert torch.equal(a, b)
        assert torch.equal(out, ref_out)


def _capture(step):
    step()                                   # warm-up outside the capture (one-time queries)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()               # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    return graph


@pytest.mark.parametrize("form", ["static", "batch", "minmax", "minmax_unrotated"])
def test_graph_replays_of_the_other_one_launch_forms(form):
    """thc_encode_all_static (no workspace argument at all), the batched pair (records
    written by argument-carrying kernels) and the one-pass min/max pair under capture:
    every replay against the eager per-bucket calls on the same inputs."""
    l, bits, W = 14, 4, 8
    ns = [40 * (1 << 14) + 77, 25 << 14] if form == "batch" else [120 * (1 << 14) + 77]
    rotate = form != "minmax_unrotated"
    if not rotate:
        ns = [ns[0] + 1]                     # an even bf16 count: the pipelined unrotated encoder
    xs = [[_rand(n, 7 + w + 50 * k) for w in range(W)] for k, n in enumerate(ns)]
    pay = [[torch.empty(thc.thc_payload_bytes(n, l, bits), dtype=torch.uint8, device=DEV) for _ in range(W)]
           for n in ns]
    per_chunk = 2 if form.startswith("minmax") else 1
    scale = [torch.empty(per_chunk * thc.thc_num_chunks(n, l), device=DEV) for n in ns]
    out = [torch.empty(n, device=DEV) for n in ns]
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    if form == "static":
        def step():
            thc.thc_encode_all_static(xs[0], l, 5, bits, pay[0], scale[0], flag)
            thc.thc_aggregate_decode(pay[0], scale[0], ns[0], l, 5, bits, None, out[0])
    elif form == "batch":
        bk = [dict(grads=xs[k], payloads=pay[k], scale=scale[k], out=out[k], n=n, seed=5 + k) for k, n in enumerate(ns)]
        ws = torch.empty(thc.thc_batch_workspace_bytes(ns, W, l), dtype=torch.uint8, device=DEV)

        def step():
            thc.thc_encode_all_batch(bk, l, bits, ws)
            thc.thc_aggregate_decode_batch(bk, l, bits, ws)
    else:
        ws = torch.empty(thc.thc_encode_all_minmax_workspace_bytes(W, ns[0], l), dtype=torch.uint8, device=DEV)

        def step():
            thc.thc_encode_all_minmax(xs[0], l, 5, bits, rotate, pay[0], scale[0], ws)
            thc.thc_aggregate_decode_minmax(pay[0], scale[0], ns[0], l, 5, bits, rotate, out[0])
    graph = _capture(step)

    for rep in range(3):
        print(f"graph replay {rep} form={form}", flush=True)
        for k in range(len(ns)):
            for w in range(W):               # new inputs in the recorded buffers
                xs[k][w].copy_(_rand(ns[k], 100 * rep + w + 50 * k))
            for p in pay[k]:
                p.fill_(0xEE)
            out[k].fill_(float("nan"))
            scale[k].fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if form == "static":
            assert int(flag.item()) == 0
        else:
            assert not thc.thc_encode_all_timed_out(ws)
        for k, n in enumerate(ns):           # eager, between replays
            ref_pay = [torch.empty_like(p) for p in pay[k]]
            ref_scale, ref_out = torch.empty_like(scale[k]), torch.empty_like(out[k])
            if form.startswith("minmax"):
                w2 = torch.empty(thc.thc_encode_all_minmax_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
                thc.thc_encode_all_minmax(xs[k], l, 5, bits, rotate, ref_pay, ref_scale, w2)
                thc.thc_aggregate_decode_minmax(ref_pay, ref_scale, n, l, 5, bits, rotate, ref_out)
            else:
                w2 = torch.empty(thc.thc_encode_all_workspace_bytes(W, n, l), dtype=torch.uint8, device=DEV)
                thc.thc_encode_all(xs[k], l, 5 + k, bits, ref_pay, ref_scale, w2)
                thc.thc_aggregate_decode(ref_pay, ref_scale, n, l, 5 + k, bits, None, ref_out)
            torch.cuda.synchronize()
            assert torch.equal(scale[k], ref_scale)
            for a, b in zip(pay[k], ref_pay):
                assert torch.equal(a, b)
            assert torch.equal(out[k], ref_out)


def test_graph_replays_of_the_full_rotation_step():
    """The full-rotation step in its deferred form (the range word is cleared by a kernel, the
    absmax atomics start from that word) under capture: every replay against eager calls."""
    l, bits, W = 17, 4, 3
    n, size = 100_001, 1 << 17
    xs = [_rand(n, 7 + w) for w in range(W)]
    work = [torch.empty(size, device=DEV) for _ in range(W)]
    absmax = torch.empty(W, device=DEV)
    scale = torch.empty(1, device=DEV)
    pay = [torch.empty(size * bits // 8, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sums = torch.empty(size, dtype=torch.uint8, device=DEV)
    out = torch.empty(n, device=DEV)

    def run(work, absmax, scale, pay, sums, out):
        for w in range(W):
            thc.rht_forward_full_deferred(xs[w], l, 5, work[w], absmax[w:w + 1])
        thc.thc_scale_reduce(absmax, W, 1, scale)
        for w in range(W):
            thc.thc_full_encode_deferred(work[w], n, l, 5, w, bits, scale, pay[w])
        thc.thc_aggregate(pay, size, 14, bits, sums)
        thc.thc_full_decode_inverse(sums, scale, W, n, l, 5, bits, work[0], out)

    graph = _capture(lambda: run(work, absmax, scale, pay, sums, out))
    ref = dict(work=[torch.empty_like(t) for t in work], absmax=torch.empty_like(absmax), scale=torch.empty_like(scale),
               pay=[torch.empty_like(p) for p in pay], sums=torch.empty_like(sums), out=torch.empty_like(out))
    for rep in range(3):
        print(f"graph replay {rep} full rotation", flush=True)
        for w in range(W):                   # new inputs in the recorded buffers
            xs[w].copy_(_rand(n, 100 * rep + w) * (10.0 ** rep))
        for p in pay:
            p.fill_(0xEE)
        out.fill_(float("nan"))
        absmax.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        run(**ref)                           # eager, between replays
        torch.cuda.synchronize()
        assert torch.equal(scale, ref["scale"]) and float(scale[0]) > 0
        for a, b in zip(pay, ref["pay"]):
            assert torch.equal(a, b)
        assert torch.equal(out, ref["out"])
