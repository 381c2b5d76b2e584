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
