#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt_1p3b] [--bits B]

One step = absmax, shared scale, encode (all W workers), aggregate and decode of
every bucket of the workload, inputs resident in HBM.  Prints ONE JSON line with
the gradient throughput (bytes of worker gradients consumed per second), the
roofline of the dominant kernel (algorithmic bytes / measured launch duration
against 8 TB/s) and the CPU oracle timed on a bounded slice of the same inputs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt_1p3b")
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=23,
                    help="coordinates per worker of the slice the CPU oracle is timed on (log2)")
    return ap.parse_args()


class Path:
    """Buffers and launch sequence of the path for one workload."""

    def __init__(self, thc, torch, wl, bits, xs, seed=0):
        self.thc, self.torch, self.wl, self.bits, self.xs, self.seed = thc, torch, wl, bits, xs, seed
        dev = xs[0].device
        self.W, self.l = wl.W, wl.chunk_log2
        self.buckets = wl.buckets()
        W, l = self.W, self.l
        self.items = []
        sb = thc.thc_sum_bytes(W, bits)
        self.sum_bytes = sb
        sum_dt = torch.uint8 if sb == 1 else torch.int16
        for k, (st, ln) in enumerate(self.buckets):
            P = thc.thc_num_chunks(ln, l)
            nb = thc.thc_payload_bytes(ln, l, bits)
            self.items.append(dict(
                st=st, ln=ln, P=P, seed=seed + k,
                grads=[x[st:st + ln] for x in xs],
                absmax=torch.empty(W * P, dtype=torch.float32, device=dev),
                scale=torch.empty(P, dtype=torch.float32, device=dev),
                payloads=[torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(W)],
                sums=torch.empty(P << l, dtype=sum_dt, device=dev),
                out=torch.empty(ln, dtype=torch.float32, device=dev)))

    def absmax(self, it):
        for w in range(self.W):
            self.thc.thc_chunk_absmax(it["grads"][w], self.l, it["seed"],
                                      it["absmax"][w * it["P"]:(w + 1) * it["P"]])
        self.thc.thc_scale_reduce(it["absmax"], self.W, it["P"], it["scale"])

    def encode(self, it):
        for w in range(self.W):
            self.thc.thc_encode(it["grads"][w], self.l, it["seed"], w, self.bits, it["scale"],
                                it["payloads"][w])

    def aggregate(self, it):
        self.thc.thc_aggregate(it["payloads"], it["ln"], self.l, self.bits, it["sums"])

    def decode(self, it):
        self.thc.thc_decode(it["sums"], it["scale"], self.W, it["ln"], self.l, it["seed"],
                            self.bits, it["out"])

    def step(self):
        for it in self.items:
            self.absmax(it)
            self.encode(it)
            self.aggregate(it)
            self.decode(it)


def time_region(torch, fn, reps):
    """Milliseconds per repetition of fn(), HIP events on the current stream."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def cpu_baseline(wl, bits, xs, log2_sample):
    """The NumPy oracle (float32 canonical-order mode), as it stands, on the first
    2^log2_sample coordinates of every worker; single process."""
    import numpy as np

    from oracle import thc as O
    from synth import to_numpy_bits
    m = min(wl.n, 1 << log2_sample)
    hx = [to_numpy_bits(x[:m]) for x in xs]
    t0 = time.perf_counter()
    O.pipeline(hx, wl.chunk_log2, 0, bits, dtype=np.float32, bf16=(wl.dtype == "bf16"))
    dt = time.perf_counter() - t0
    s_in = 2 if wl.dtype == "bf16" else 4
    return dict(value=wl.W * m * s_in / dt / 1e9, unit="GB/s", cores=1, kind="oracle",
                sample=f"first 2^{log2_sample} coordinates of each of the {wl.W} workers "
                       f"({dt:.1f} s of NumPy, one thread)")


def read_traffic(workload_name, bits):
    """HBM bytes per launch of the dominant kernel, measured offline with rocprofv3
    --pmc (FETCH_SIZE, WRITE_SIZE) and kept in profiles/hbm_traffic.txt as lines
    `<workload> <bits> <kernel> <bytes_per_launch>`."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 4 and not line.startswith("#") and f[0] == workload_name and f[1] == str(bits):
            return float(f[3])
    return None


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (W workers are simulated in one GPU's "
              "memory; there are no collectives).  Run with --gpus 1.", file=sys.stderr)
        return 2
    import torch

    import paper_2407_01378_amd as thc
    from synth import generate, workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    thc.lib()
    dev = torch.device("cuda:0")
    wl = workload(a.workload)
    bits = a.bits if a.bits is not None else wl.bits[0]
    s_in = 2 if wl.dtype == "bf16" else 4

    xs = [generate(wl, w, dev) for w in range(wl.W)]
    path = Path(thc, torch, wl, bits, xs)
    torch.cuda.synchronize()

    for _ in range(a.warmup):
        path.step()
    ms = time_region(torch, path.step, a.steps)

    # per-kernel launch durations, live, on the same stream
    def all_items(fn):
        def run():
            for it in path.items:
                fn(it)
        return run
    kernels = {}
    launches = {"absmax": wl.W * len(path.items), "encode": wl.W * len(path.items),
                "aggregate": len(path.items), "decode": len(path.items)}
    for name, fn in (("absmax", path.absmax), ("encode", path.encode),
                     ("aggregate", path.aggregate), ("decode", path.decode)):
        t = time_region(torch, all_items(fn), max(2, a.steps // 2))
        kernels[name] = dict(ms_per_step=round(t, 4), us_per_launch=round(1e3 * t / launches[name], 3))

    # dominant kernel: thc_encode (W launches per bucket).  Algorithmic bytes per
    # worker-coordinate: the gradient read once + its payload written once.
    n_total = wl.n
    enc_bytes_per_launch = (n_total / len(path.items)) * (s_in + bits / 8.0)
    enc_s = kernels["encode"]["us_per_launch"] * 1e-6
    achieved = enc_bytes_per_launch / enc_s / 1e9
    traffic = read_traffic(wl.name, bits)

    sb = path.sum_bytes
    alg_bytes_per_coord = wl.W * (s_in + bits / 8.0) + wl.W * bits / 8.0 + 2 * sb + 4
    value = wl.W * wl.n * s_in / (ms * 1e-3) / 1e9
    res = {
        "metric": "gradient GB/s for encode+aggregate+decode (W workers), 1 GPU",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": wl.W, "n": wl.n, "input": wl.dtype, "bits": bits,
                   "chunk_log2": wl.chunk_log2, "buckets": len(path.items),
                   "bucket_elems": wl.bucket or wl.n},
        "roofline": {"bound": "hbm", "kernel": "thc_encode", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic},
        "pipeline_hbm": {"algorithmic_bytes_per_coord": alg_bytes_per_coord,
                         "achieved_GBps": round(wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "kernels": kernels,
    }
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, bits, xs, a.cpu_sample_log2)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
