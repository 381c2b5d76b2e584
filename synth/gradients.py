"""Seeded synthetic gradients shaped like the paper's training workloads.

The paper measures on VGG19 / TinyImageNet and BERT-large / WikiText-103; those
models, datasets and their real gradients are not available here, so these
generators stand in for them: flattened per-worker gradients with the layer
structure, sizes, value distributions and sparsity of five named workloads.
This module is the ONLY code shared by the CPU oracle's tests and the GPU
library's tests; it contains none of the method's arithmetic (no rotation, no
quantizer, no Philox) - just torch's own seeded generators.

Layout: every worker's gradient is one contiguous 1-D tensor of `n` elements,
made of consecutive segments (layers).  The segment table (sizes, scales) is
drawn once per workload from numpy's default_rng(workload id) and is the same
for all workers; the values are drawn per worker from a torch.Generator seeded
with 1000 * workload id + worker, segment after segment in order.
"""

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np
import torch


@dataclass
class Segment:
    size: int
    kind: str        # "normal" | "student3" | "sparse_rows"
    scale: float
    row: int = 0     # row length for "sparse_rows"
    p_zero: float = 0.0


@dataclass
class Workload:
    name: str
    wid: int
    W: int
    dtype: str                 # "f32" | "bf16"
    n: int
    chunk_log2: int
    bits: Tuple[int, ...]
    bucket: int                # elements per DDP-style bucket (0 = one bucket)
    segments: List[Segment] = field(default_factory=list)

    def buckets(self):
        """[(start, length)] covering [0, n) in order."""
        if not self.bucket:
            return [(0, self.n)]
        out, s = [], 0
        while s < self.n:
            ln = min(self.bucket, self.n - s)
            out.append((s, ln))
            s += ln
        return out


def _loguniform(rng, lo, hi, k):
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=k))


def _transformer_layer(h, ffn):
    return h * 3 * h + h * h + h * ffn + ffn * h + 4 * h


def workload(name: str) -> Workload:
    if name == "tiny":
        rng = np.random.default_rng(1)
        f = _loguniform(rng, 1e-4, 1e-1, 16)
        segs = [Segment(1 << 16, "normal", float(s)) for s in f]
        return Workload(name, 1, 4, "f32", 1 << 20, 10, (4,), 0, segs)
    if name == "resnet50":
        rng = np.random.default_rng(2)
        n = 25_557_032
        w = _loguniform(rng, 64.0, 2.4e6, 161)
        sizes = np.floor(n * w / w.sum()).astype(np.int64)
        sizes[-1] += n - sizes.sum()
        sig = _loguniform(rng, 1e-5, 1e-2, 161)
        segs = [Segment(int(z), "normal", float(s)) for z, s in zip(sizes, sig)]
        return Workload(name, 2, 8, "f32", n, 14, (4,), 0, segs)
    if name == "bert_base":
        segs = [Segment(30522 * 768, "sparse_rows", 1e-3, row=768, p_zero=0.99)]
        segs += [Segment(_transformer_layer(768, 3072), "student3", 1e-3) for _ in range(12)]
        n = sum(s.size for s in segs)
        assert n == 108_412_416
        return Workload(name, 3, 8, "bf16", n, 14, (4,), 0, segs)
    if name == "gpt_345m":
        rng = np.random.default_rng(4)
        sc = _loguniform(rng, 1e-5, 1e-2, 25)
        segs = [Segment(50257 * 1024, "student3", float(sc[0]))]
        segs += [Segment(_transformer_layer(1024, 4096), "student3", float(s)) for s in sc[1:]]
        n = sum(s.size for s in segs)
        assert n == 353_551_360
        return Workload(name, 4, 8, "bf16", n, 14, (2, 8), 0, segs)
    if name == "gpt_1p3b":
        rng = np.random.default_rng(5)
        sc = _loguniform(rng, 1e-5, 1e-2, 25)
        per = _transformer_layer(2048, 8192)
        assert per == 50_339_840
        segs = [Segment(per, "student3", float(s)) for s in sc[:24]]
        n = 1_300_000_000
        segs.append(Segment(n - 24 * per, "student3", float(sc[24])))
        return Workload(name, 5, 8, "bf16", n, 14, (4,), 25 * (1 << 20), segs)
    raise KeyError(name)


WORKLOADS = ("tiny", "resnet50", "bert_base", "gpt_345m", "gpt_1p3b")


def _student3(m, gen, device):
    z = torch.randn(4, m, generator=gen, device=device, dtype=torch.float32)
    chi = (z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0
    return z[0] / torch.sqrt(chi)


def generate(wl: Workload, worker: int, device="cpu", max_elems=None) -> torch.Tensor:
    """Worker `worker`'s flattened gradient (fp32 or bf16 tensor of wl.n elements,
    or a shorter stand-in of max_elems elements with the same leading segment
    structure - a fresh, shorter draw per segment, not a prefix of the full one)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(1000 * wl.wid + worker)
    n = wl.n if max_elems is None else min(wl.n, int(max_elems))
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    out = torch.empty(n, dtype=tdt, device=device)
    pos = 0
    for seg in wl.segments:
        if pos >= n:
            break
        take = min(seg.size, n - pos)
        if seg.kind == "normal":
            v = torch.randn(take, generator=gen, device=device, dtype=torch.float32) * seg.scale
        elif seg.kind == "student3":
            v = _student3(take, gen, device) * seg.scale
        elif seg.kind == "sparse_rows":
            rows = (take + seg.row - 1) // seg.row
            keep = torch.rand(rows, generator=gen, device=device) >= seg.p_zero
            v = _student3(rows * seg.row, gen, device) * seg.scale
            v = (v.view(rows, seg.row) * keep.view(rows, 1).to(v.dtype)).view(-1)
        else:
            raise ValueError(seg.kind)
        out[pos:pos + take] = v[:take].to(tdt)
        pos += take
        del v
    assert pos == n
    return out


def to_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy in the form the oracle takes: float32 array, or the uint16 bit
    patterns of a bf16 tensor."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()
