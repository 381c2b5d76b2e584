#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt_1p3b] [--bits B]
                    [--unfused]

One step = every bucket of the workload through the whole path, inputs resident in
HBM: rotation, shared per-chunk scale, stochastic rounding + packing of all W
workers (thc_encode_all), then integer aggregation, dequantization and inverse
rotation (thc_aggregate_decode).  --unfused times the one-call-per-step form
(thc_chunk_absmax, thc_scale_reduce, thc_encode, thc_aggregate, thc_decode) instead.

Prints ONE JSON line: gradient throughput (bytes of worker gradients consumed per
second), the roofline of the dominant kernel (algorithmic bytes per launch / measured
launch duration against 8 TB/s; the same kernel's algorithmic arithmetic against the
plain-VALU issue rate is given beside it), and the CPU oracle timed on a bounded slice
of the same inputs.

    python bench.py --sat        the saturation-based aggregation variant (signed 2^b - 1 level
                                 grid, Sat in worker order, b-bit aggregate); also reports the
                                 overflow rate and the vNMSE next to the exact-sum path's
    python bench.py --full-rotation   the paper's baseline: one rotation over the whole gradient
                                 padded to 2^l (rotated data goes through HBM; separate
                                 range / encode / aggregate / decode calls); no buckets
    python bench.py --quality    vNMSE and time of one bucket for the grid / rotation variants:
                                 symmetric range + partial rotation (the timed path), min/max
                                 range + partial rotation, min/max range without rotation
    python bench.py --topkc      the paper's TopK Chunked sparsifier on the same gradients
                                 (C = 64, J for about 2 bits per coordinate): time per step,
                                 norm-kernel roofline, vNMSE
    python bench.py --probe      a few launches of each kernel of the first bucket plus a
                                 device-to-device copy of known size; meant to run under
                                 rocprofv3 --pmc so that counter readings of the kernels
                                 can be scaled by what the same counter reads for the copy
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
# Plain (unpacked, unfused) VALU issue rate: 256 CUs x 4 SIMDs x 16 lanes per clock at
# 2.4 GHz.  The published 157.3 TFLOP/s fp32 vector figure is this rate x 2 (FMA) x 2
# (packed fp32); the path's separately rounded adds, subtracts and integer ops can use
# neither.
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
# Arithmetic the method asks for per worker-coordinate of the encode step at chunk 2^14:
# sign flip, 14 butterfly stages, range, five quantizer ops (random byte to float, noise
# constant, fused position + noise, floor, pack; the normalisation folds into the
# multiplier), and one Philox4x32-10 block (10 rounds of 2 wide multiplies + 2 three-input
# xors, 18 key additions) per 16 coordinates.
ENCODE_OPS_PER_COORD = 1 + 14 + 1 + 5 + (10 * 4 + 18) / 16.0
PROBE_COPY_BYTES = 1 << 29


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt_1p3b")
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--unfused", action="store_true")
    ap.add_argument("--sat", action="store_true", help="saturation-based aggregation variant")
    ap.add_argument("--full-rotation", action="store_true",
                    help="full rotation baseline (l' = l) instead of the chunked path")
    ap.add_argument("--quality", action="store_true",
                    help="vNMSE / time comparison of the range and rotation variants on one bucket")
    ap.add_argument("--topkc", action="store_true", help="TopK Chunked sparsifier instead of THC")
    ap.add_argument("--topkc-chunk", type=int, default=64)
    ap.add_argument("--topkc-bits", type=float, default=2.0, help="target bits per coordinate")
    ap.add_argument("--workers", type=int, default=None,
                    help="simulate this many workers instead of the workload's own W")
    ap.add_argument("--first-buckets", type=int, default=None,
                    help="keep only the first K buckets of every worker's gradient (quality runs "
                         "with many workers; not the headline configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe", action="store_true",
                    help="few launches + a copy of known size, for rocprofv3 --pmc runs")
    ap.add_argument("--cpu-sample-log2", type=int, default=25,
                    help="coordinates per worker of the slice the CPU oracle is timed on (log2)")
    return ap.parse_args()


class Path:
    """Buffers and launch sequence of the path for one workload."""

    def __init__(self, thc, torch, wl, bits, xs, seed=0, fused=True, sat=False):
        self.thc, self.wl, self.bits, self.fused, self.sat = thc, wl, bits, fused, sat
        assert fused or not sat, "--sat is timed in its fused form"
        self.overflow = torch.zeros(1, dtype=torch.int64, device=xs[0].device)
        self.count_overflow = False   # the timed steps run without the optional overflow counter
        dev = xs[0].device
        self.W, self.l = wl.W, wl.chunk_log2
        W, l = self.W, self.l
        self.items = []
        self.sum_bytes = thc.thc_sum_bytes(W, bits)
        sum_dt = torch.uint8 if self.sum_bytes == 1 else torch.int16
        self.no_sums = fused and (thc.thc_sat_aggregate_decode_is_fused(W, l, bits) if sat
                                  else thc.thc_aggregate_decode_is_fused(W, l, bits))
        assert self.no_sums or not sat, "--sat needs a shape whose aggregate+decode runs fused"
        for k, (st, ln) in enumerate(wl.buckets()):
            P = thc.thc_num_chunks(ln, l)
            nb = thc.thc_payload_bytes(ln, l, bits)
            it = dict(st=st, ln=ln, P=P, seed=seed + k,
                      grads=[x[st:st + ln] for x in xs],
                      scale=torch.empty(P, dtype=torch.float32, device=dev),
                      payloads=[torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(W)],
                      out=torch.empty(ln, dtype=torch.float32, device=dev))
            if fused:
                # one workspace per bucket, cleared once: the timed calls are the form that
                # expects it clear and leaves it clear (no clearing launch per call)
                it["ws"] = torch.empty(thc.thc_encode_all_workspace_bytes(W, ln, l),
                                       dtype=torch.uint8, device=dev)
                thc.thc_workspace_clear(it["ws"])
            else:
                it["absmax"] = torch.empty(W * P, dtype=torch.float32, device=dev)
            it["sums"] = None if self.no_sums else torch.empty(P << l, dtype=sum_dt, device=dev)
            self.items.append(it)
        if fused:
            self.phases = {"encode_all": (self.encode_all, 1), "aggregate_decode": (self.aggregate_decode, 1)}
            self.dominant = "encode_all"
        else:
            self.phases = {"absmax": (self.absmax, W), "encode": (self.encode, W),
                           "aggregate": (self.aggregate, 1), "decode": (self.decode, 1)}
            self.dominant = "encode"

    # fused form
    def encode_all(self, it):
        fn = self.thc.thc_sat_encode_all_cleared if self.sat else self.thc.thc_encode_all_cleared
        fn(it["grads"], self.l, it["seed"], self.bits, it["payloads"], it["scale"], it["ws"])

    def aggregate_decode(self, it):
        if self.sat:
            self.thc.thc_sat_aggregate_decode(it["payloads"], it["scale"], it["ln"], self.l,
                                              it["seed"], self.bits, None,
                                              self.overflow if self.count_overflow else None, it["out"])
        else:
            self.thc.thc_aggregate_decode(it["payloads"], it["scale"], it["ln"], self.l, it["seed"],
                                          self.bits, it["sums"], it["out"])

    # one call per step of the method
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
            for fn, _ in self.phases.values():
                fn(it)

    def timed_out(self):
        return self.fused and any(self.thc.thc_encode_all_timed_out(it["ws"]) for it in self.items)


class FullPath:
    """The same method with ONE rotation over the whole gradient (l' = l)."""

    def __init__(self, thc, torch, wl, bits, xs):
        self.thc, self.torch, self.wl, self.bits, self.xs = thc, torch, wl, bits, xs
        dev = xs[0].device
        self.W, self.n = wl.W, wl.n
        self.l = thc.thc_full_log2(wl.n)
        size = 1 << self.l
        self.size = size
        self.ys = [torch.empty(size, dtype=torch.float32, device=dev) for _ in range(self.W)]
        self.absmax = torch.empty(self.W, dtype=torch.float32, device=dev)
        self.scale = torch.empty(1, dtype=torch.float32, device=dev)
        self.payloads = [torch.empty(size * bits // 8, dtype=torch.uint8, device=dev) for _ in range(self.W)]
        self.sum_bytes = thc.thc_sum_bytes(self.W, bits)
        self.sums = torch.empty(size, dtype=torch.uint8 if self.sum_bytes == 1 else torch.int16, device=dev)
        self.out = torch.empty(self.n, dtype=torch.float32, device=dev)
        self.fused, self.sat = False, False
        self.phases = {"rht_forward_full_deferred": (self.rotate, self.W), "scale_reduce": (self.ranges, 1),
                       "full_encode_deferred": (self.encode, self.W), "aggregate": (self.aggregate, 1),
                       "full_decode_inverse": (self.decode_inverse, 1)}
        self.dominant = "rht_forward_full_deferred"
        self.items = [None]

    def rotate(self, _=None):
        for w in range(self.W):
            self.thc.rht_forward_full_deferred(self.xs[w], self.l, 0, self.ys[w], self.absmax[w:w + 1])

    def ranges(self, _=None):
        self.thc.thc_scale_reduce(self.absmax, self.W, 1, self.scale)

    def encode(self, _=None):
        for w in range(self.W):
            self.thc.thc_full_encode_deferred(self.ys[w], self.n, self.l, 0, w, self.bits, self.scale,
                                              self.payloads[w])

    def aggregate(self, _=None):
        self.thc.thc_aggregate(self.payloads, self.size, 14, self.bits, self.sums)

    def decode_inverse(self, _=None):
        self.thc.thc_full_decode_inverse(self.sums, self.scale, self.W, self.n, self.l, 0, self.bits,
                                         self.ys[0], self.out)

    def step(self):
        for fn, _ in self.phases.values():
            fn()

    def timed_out(self):
        return False


def time_steps(torch, fn, steps):
    """Exactly `steps` repetitions of fn(), bracketed by synchronisation on both sides, with
    one HIP event between consecutive repetitions (no synchronisation in between).
    Returns (median, mean, min, max) of the per-step times in milliseconds."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    med = t[steps // 2] if steps % 2 else 0.5 * (t[steps // 2 - 1] + t[steps // 2])
    return med, ev[0].elapsed_time(ev[steps]) / steps, t[0], t[-1]


_POOL_INPUT = None


def _oracle_pool_init(shm_name, W, m, np_dtype):
    """Pool initializer of the all-cores leg: map the parent's copy of the sample."""
    global _POOL_INPUT
    from multiprocessing import shared_memory

    import numpy as np
    shm = shared_memory.SharedMemory(name=shm_name)
    _POOL_INPUT = (shm, np.ndarray((W, m), dtype=np.dtype(np_dtype), buffer=shm.buf))


def _oracle_slice(args):
    """Pool worker of the all-cores leg: the oracle on one slice (whole chunks) of every
    worker's sample."""
    import numpy as np

    from oracle import thc as O
    g0, piece, chunk_log2, bits, bf16 = args
    x = _POOL_INPUT[1]
    O.pipeline([x[w, g0:g0 + piece] for w in range(x.shape[0])], chunk_log2, 0, bits,
               dtype=np.float32, bf16=bf16, g0=g0)
    return piece


def cpu_baseline(wl, bits, xs, log2_sample):
    """The NumPy oracle (float32 canonical-order mode), as it stands, on the first coordinates
    of every worker: once in this process (NumPy runs these operations on one thread), once
    with a process pool over slices of whole chunks on the host cores this job may use."""
    import numpy as np

    from oracle import thc as O
    from synth import to_numpy_bits
    s_in = 2 if wl.dtype == "bf16" else 4
    bf16 = wl.dtype == "bf16"
    m = min(wl.n, 1 << log2_sample)
    hx = [to_numpy_bits(x[:m]) for x in xs]
    t0 = time.perf_counter()
    O.pipeline(hx, wl.chunk_log2, 0, bits, dtype=np.float32, bf16=bf16)
    dt = time.perf_counter() - t0
    res = dict(value=round(wl.W * m * s_in / dt / 1e9, 5), unit="GB/s", cores=1, kind="oracle",
               sample=f"first 2^{log2_sample} coordinates of each of the {wl.W} workers "
                      f"({dt:.1f} s of NumPy, one thread)")
    # all cores: the job's share of the host is 16 threads whatever the machine reports
    cores = max(1, min(os.cpu_count() or 1, 16))
    piece = 1 << 21                              # 128 chunks of 2^14 per task
    m_all = min(wl.n, max(m, piece * cores * 2)) // piece * piece
    if cores > 1 and m_all >= 2 * piece:
        try:
            res["all_cores"] = _cpu_baseline_pool(wl, bits, xs, m_all, piece, cores, bf16, s_in)
        except Exception as e:   # the reported baseline must not take the GPU measurement down with it
            res["all_cores"] = dict(error=f"{type(e).__name__}: {e}", cores=cores, host_cpu_count=os.cpu_count())
    return res


def _cpu_baseline_pool(wl, bits, xs, m_all, piece, cores, bf16, s_in):
    """The all-cores leg: the sample in shared memory, a spawned process pool over its slices."""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    from multiprocessing import shared_memory

    import numpy as np

    from synth import to_numpy_bits
    first = to_numpy_bits(xs[0][:m_all])
    shm = shared_memory.SharedMemory(create=True, size=wl.W * m_all * first.itemsize)
    try:
        host = np.ndarray((wl.W, m_all), dtype=first.dtype, buffer=shm.buf)
        host[0] = first
        for w in range(1, wl.W):
            host[w] = to_numpy_bits(xs[w][:m_all])
        tasks = [(g, piece, wl.chunk_log2, bits, bf16) for g in range(0, m_all, piece)]
        ctx = mp.get_context("spawn")            # the parent holds a GPU context: no fork
        # an executor, not multiprocessing.Pool: a worker that dies ends the leg with an
        # error instead of being replaced for ever
        with ProcessPoolExecutor(cores, mp_context=ctx, initializer=_oracle_pool_init,
                                 initargs=(shm.name, wl.W, m_all, first.dtype.str)) as pool:
            list(pool.map(_oracle_slice,
                          [(0, 1 << wl.chunk_log2, wl.chunk_log2, bits, bf16)] * cores))   # start-up, untimed
            t0 = time.perf_counter()
            done = sum(pool.map(_oracle_slice, tasks))
            dt_all = time.perf_counter() - t0
        del host
    finally:
        shm.close()
        shm.unlink()
    return dict(value=round(wl.W * done * s_in / dt_all / 1e9, 5), unit="GB/s", cores=cores,
                host_cpu_count=os.cpu_count(),
                kind="oracle, process pool over slices of 2^21 coordinates",
                sample=f"first {done} coordinates of each of the {wl.W} workers ({dt_all:.1f} s wall)")


def copy_bandwidth(torch, dev):
    """GB/s of HBM traffic (read + write) of a plain device-to-device copy of 1 GiB."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    ms = time_steps(torch, lambda: dst.copy_(src), 10)[0]
    return 2.0 * src.numel() * 4 / (ms * 1e-3) / 1e9


def probe(torch, path, dev):
    """Three launches of every kernel of the first bucket and three copies of
    PROBE_COPY_BYTES bytes (one elementwise kernel each)."""
    it = path.items[0]
    src = torch.empty(PROBE_COPY_BYTES // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        for fn, _ in path.phases.values():
            fn(it)
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"probe": "ok", "bucket_elems": it["ln"] if it else None, "copy_bytes": PROBE_COPY_BYTES}))


def vnmse(torch, path, it):
    """||estimate - mean||^2 / ||mean||^2 of one bucket, the error measure of the paper's
    evaluation section, with the exact fp32 mean of the W workers' gradients as reference."""
    mean = torch.zeros(it["ln"], dtype=torch.float32, device=it["out"].device)
    for g in it["grads"]:
        mean += g.float()
    mean /= len(it["grads"])
    return float(((it["out"] - mean) ** 2).sum() / (mean ** 2).sum())


def quality(thc, torch, wl, bits, xs, dev):
    """One bucket through three variants of the method; vNMSE against the exact fp32 mean
    and milliseconds per pass (HIP events, 5 repetitions after one warm-up)."""
    st, ln = wl.buckets()[0]
    W, l = wl.W, wl.chunk_log2
    grads = [x[st:st + ln] for x in xs]
    P = thc.thc_num_chunks(ln, l)
    nb = thc.thc_payload_bytes(ln, l, bits)
    sb = thc.thc_sum_bytes(W, bits)
    payloads = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(W)]
    sums = torch.empty(P << l, dtype=torch.uint8 if sb == 1 else torch.int16, device=dev)
    out = torch.empty(ln, dtype=torch.float32, device=dev)
    scale = torch.empty(P, dtype=torch.float32, device=dev)
    ws = torch.empty(thc.thc_encode_all_workspace_bytes(W, ln, l), dtype=torch.uint8, device=dev)
    ranges_all = torch.empty(W * P * 2, dtype=torch.float32, device=dev)
    rng = torch.empty(P * 2, dtype=torch.float32, device=dev)
    mean = torch.zeros(ln, dtype=torch.float32, device=dev)
    for g in grads:
        mean += g.float()
    mean /= W

    def symmetric():
        thc.thc_encode_all(grads, l, 0, bits, payloads, scale, ws)
        thc.thc_aggregate_decode(payloads, scale, ln, l, 0, bits, sums, out)

    def minmax(rotate):
        for w in range(W):
            thc.thc_chunk_minmax(grads[w], l, 0, rotate, ranges_all[2 * w * P:2 * (w + 1) * P])
        thc.thc_range_reduce(ranges_all, W, P, rng)
        for w in range(W):
            thc.thc_encode_minmax(grads[w], l, 0, w, bits, rotate, rng, payloads[w])
        thc.thc_aggregate(payloads, ln, l, bits, sums)
        thc.thc_decode_minmax(sums, rng, W, ln, l, 0, bits, rotate, out)

    ws_mm = torch.empty(thc.thc_encode_all_minmax_workspace_bytes(W, ln, l), dtype=torch.uint8, device=dev) \
        if l == 14 and thc.thc_aggregate_decode_is_fused(W, l, bits) else None

    def minmax_one_pass(rotate):
        thc.thc_encode_all_minmax(grads, l, 0, bits, rotate, payloads, rng, ws_mm)
        thc.thc_aggregate_decode_minmax(payloads, rng, ln, l, 0, bits, rotate, out)

    variants = [("symmetric_partial_rotation", symmetric)]
    if ws_mm is not None:
        variants += [("minmax_partial_rotation", lambda: minmax_one_pass(True)),
                     ("minmax_no_rotation", lambda: minmax_one_pass(False))]
    variants += [("minmax_partial_rotation_per_step_calls", lambda: minmax(True)),
                 ("minmax_no_rotation_per_step_calls", lambda: minmax(False))]
    res = {}
    for name, fn in variants:
        fn()
        ms = time_steps(torch, fn, 5)[0]
        err = float(((out - mean) ** 2).sum() / (mean ** 2).sum())
        res[name] = {"vnmse": err, "ms_per_bucket": round(ms, 4),
                     "gradient_GBps": round(W * ln * (2 if wl.dtype == "bf16" else 4) / (ms * 1e-3) / 1e9, 1)}
    return {"workload": wl.name, "bucket_elems": ln, "W": W, "bits": bits, "variants": res}


def topkc_bench(thc, torch, wl, xs, dev, a):
    """Whole TopKC round on the full gradient of every worker (no buckets: the selection is
    global): norms x W, fp16 sum, selection, fp16 chunk sums, dense estimate."""
    W, n, C = wl.W, wl.n, a.topkc_chunk
    s_in = 2 if wl.dtype == "bf16" else 4
    P = thc.topkc_num_chunks(n, C)
    J = max(1, int((a.topkc_bits / 16.0 - 1.0 / C) * n / C))
    norms_all = torch.empty(W * P, dtype=torch.float16, device=dev)
    s = torch.empty(P, dtype=torch.float16, device=dev)
    idx = torch.empty(J, dtype=torch.int32, device=dev)
    ws = torch.empty(thc.topkc_select_workspace_bytes(P), dtype=torch.uint8, device=dev)
    vals = torch.empty(J * C, dtype=torch.float16, device=dev)
    out = torch.empty(n, dtype=torch.float32, device=dev)

    def norms():
        for w in range(W):
            thc.topkc_chunk_norms(xs[w], C, norms_all[w * P:(w + 1) * P])

    phases = {"chunk_norms": (norms, W),
              "sum_norms": (lambda: thc.topkc_sum_norms(norms_all, W, P, s), 1),
              "select": (lambda: thc.topkc_select(s, J, idx, ws), 1),
              "gather_sum": (lambda: thc.topkc_gather_sum(xs, C, idx, J, vals), 1),
              "scatter_mean": (lambda: thc.topkc_scatter_mean(vals, idx, J, C, W, out), 1)}

    def step():
        for fn, _ in phases.values():
            fn()

    step()
    torch.cuda.synchronize()
    t_end = time.perf_counter() + 0.5
    while time.perf_counter() < t_end:
        step()
        torch.cuda.synchronize()
    for _ in range(a.warmup):
        step()
    ms = time_steps(torch, step, a.steps)[0]
    kernels = {}
    for name, (fn, calls) in phases.items():
        t = time_steps(torch, fn, max(3, a.steps // 2))[0]
        kernels[name] = dict(ms_per_step=round(t, 4), launches_per_step=calls,
                             us_per_launch=round(1e3 * t / calls, 3))
    step()
    torch.cuda.synchronize()
    mean = torch.zeros(n, dtype=torch.float32, device=dev)
    for x in xs:
        mean += x.float()
    mean /= W
    err = float(((out - mean) ** 2).sum() / (mean ** 2).sum())
    dom_bytes = n * s_in + P * 2                      # one norms launch: gradient in, fp16 norms out
    dom_s = kernels["chunk_norms"]["us_per_launch"] * 1e-6
    achieved = dom_bytes / dom_s / 1e9
    # what the method must move per coordinate: every gradient read for the norms, the
    # selected chunks read again and their fp16 sum written, the dense estimate written
    frac = J * C / n
    alg = W * s_in + W * s_in * frac + 2 * frac + 4 + (W + 2) * 2.0 / C
    return {
        "metric": "gradient GB/s for TopKC (norms + select + chunk sums + estimate, W workers), 1 GPU",
        "value": round(W * n * s_in / (ms * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "W": W, "n": n, "input": wl.dtype, "method": "topkc", "C": C, "J": J,
                   "bits_per_coordinate": round(16.0 * (J * C / n + 1.0 / C), 4)},
        "roofline": {"bound": "hbm", "kernel": "topkc_chunk_norms", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": read_traffic(wl.name, "f16", "topkc_chunk_norms") if (C, W) == (64, 8) else None},
        "pipeline_hbm": {"algorithmic_bytes_per_coord": round(alg, 3),
                         "achieved_GBps": round(n * alg / (ms * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(n * alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "vnmse": err, "kernels": kernels,
    }


def read_traffic(workload_name, bits, kernel):
    """HBM bytes per launch of a kernel, measured offline with rocprofv3 --pmc
    (FETCH_SIZE, WRITE_SIZE) and kept in profiles/hbm_traffic.txt as lines
    `<workload> <bits> <kernel> <bytes_per_launch>`."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if (len(f) >= 4 and not line.startswith("#") and f[0] == workload_name
                and f[1] == str(bits) and f[2] == kernel):
            return float(f[3])
    return None


def read_executed_ops(workload_name, bits):
    """VALU lane-operations per worker-coordinate that the one-pass encoder executed when it
    was last counted with rocprofv3 --pmc SQ_INSTS_VALU (first bucket of the headline
    workload; profiles/encode_all_aggregate_decode_gpt_1p3b_sq_counters.txt)."""
    path = os.path.join(ROOT, "profiles", "encode_all_aggregate_decode_gpt_1p3b_sq_counters.txt")
    if workload_name != "gpt_1p3b" or bits != 4 or not os.path.exists(path):
        return None
    seen_kernel = False
    for line in open(path):
        if line.startswith("encode_all_kernel"):
            seen_kernel = True
        if seen_kernel and line.strip().startswith("all VALU"):
            return float(line.split()[-1])
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
    if a.workers is not None:
        import dataclasses
        wl = dataclasses.replace(wl, W=a.workers)
    bits = a.bits if a.bits is not None else wl.bits[0]
    s_in = 2 if wl.dtype == "bf16" else 4
    W = wl.W

    if a.first_buckets:
        keep = min(wl.n, a.first_buckets * (wl.bucket or wl.n))
        xs = [generate(wl, w, dev)[:keep].clone() for w in range(W)]
        import dataclasses
        wl = dataclasses.replace(wl, n=keep, name=f"{wl.name}[first {a.first_buckets} buckets]")
    else:
        xs = [generate(wl, w, dev) for w in range(W)]
    if a.quality:
        print(json.dumps(quality(thc, torch, wl, bits, xs, dev)))
        return 0
    if a.topkc:
        print(json.dumps(topkc_bench(thc, torch, wl, xs, dev, a)))
        return 0
    if a.full_rotation:
        path = FullPath(thc, torch, wl, bits, xs)
    else:
        path = Path(thc, torch, wl, bits, xs, fused=not a.unfused, sat=a.sat)
    torch.cuda.synchronize()
    if a.probe:
        probe(torch, path, dev)
        return 0

    # Setup, untimed: first touch of every buffer and time for the device to leave its
    # idle power state (the first ~100 ms of work after start-up run at lower clocks).
    path.step()
    torch.cuda.synchronize()
    t_end = time.perf_counter() + 0.5
    while time.perf_counter() < t_end:
        path.step()
        torch.cuda.synchronize()

    for _ in range(a.warmup):
        path.step()
    ms, ms_mean, ms_min, ms_max = time_steps(torch, path.step, a.steps)
    assert not path.timed_out(), "a bounded wait inside thc_encode_all expired"

    # per-kernel launch durations, live, on the same stream
    kernels = {}
    nb = len(path.items)
    for name, (fn, per_bucket) in path.phases.items():
        def run(fn=fn):
            for it in path.items:
                fn(it)
        t = time_steps(torch, run, max(3, a.steps // 2))[0]   # median: one disturbed repetition must not show
        kernels[name] = dict(ms_per_step=round(t, 4), launches_per_step=nb * per_bucket,
                             us_per_launch=round(1e3 * t / (nb * per_bucket), 3))

    # The same launches timed inside whole steps (an event after every phase of every bucket):
    # a kernel that reads what the previous one just wrote finds part of it in the 256 MB
    # last-level cache, so its duration there differs from that of the back-to-back loop above.
    if not a.full_rotation:
        per_rep = {name: [] for name in path.phases}
        for _ in range(3):
            evs = [torch.cuda.Event(enable_timing=True)]
            torch.cuda.synchronize()
            evs[0].record()
            for it in path.items:
                for fn, _ in path.phases.values():
                    fn(it)
                    evs.append(torch.cuda.Event(enable_timing=True))
                    evs[-1].record()
            torch.cuda.synchronize()
            tot = dict.fromkeys(path.phases, 0.0)
            for i, name in enumerate(list(path.phases) * nb):
                tot[name] += evs[i].elapsed_time(evs[i + 1])
            for name in tot:
                per_rep[name].append(tot[name])
        for name, (_, per_bucket) in path.phases.items():
            kernels[name]["us_per_launch_in_step"] = round(1e3 * sorted(per_rep[name])[1] / (nb * per_bucket), 3)

    # Dominant kernel and its algorithmic bytes per launch.  Per worker-coordinate the
    # encode step must read the gradient once and write its payload once.
    coords_per_launch = wl.n / nb
    if a.full_rotation:
        # one rht_forward_full_deferred call: gradient in, rotated fp32 chunks out, then every
        # high pass reads the part of the array that holds values (the zero padding behind the
        # gradient is implied, not stored) and writes the blocks of 2^(s0 + m) floats those
        # values reach; the last pass only reads: it is evaluated for the range, and again,
        # for the payload, by thc_full_encode_deferred
        high = path.l - 14
        valid = ((wl.n + (1 << 14) - 1) >> 14) << 14
        dom_bytes = wl.n * s_in + valid * 4
        passes, s0 = (high + 8) // 9, 14
        for p in range(passes):
            m = (path.l - s0 + (passes - p) - 1) // (passes - p)
            block = 1 << (s0 + m)
            reach = min(path.size, (valid + block - 1) // block * block)
            dom_bytes += valid * 4 + (0 if p + 1 == passes else reach) * 4
            valid, s0 = reach, s0 + m
        dom_name = "rht_forward_full_deferred"
    elif path.fused:
        dom_bytes = coords_per_launch * W * (s_in + bits / 8.0)
        dom_name = "thc_encode_all"
    else:
        dom_bytes = coords_per_launch * (s_in + bits / 8.0)
        dom_name = "thc_encode"
    dom_s = kernels[path.dominant]["us_per_launch"] * 1e-6
    achieved = dom_bytes / dom_s / 1e9

    # The other kernel of the fused form, same accounting: W payloads in, fp32 estimate out.
    second = None
    if path.fused and not a.full_rotation and "aggregate_decode" in kernels:
        sec_bytes = coords_per_launch * (W * bits / 8.0 + 4.0)
        sec_gbs = sec_bytes / (kernels["aggregate_decode"]["us_per_launch"] * 1e-6) / 1e9
        sec_name = "thc_sat_aggregate_decode" if a.sat else "thc_aggregate_decode"
        second = {"bound": "hbm", "kernel": sec_name, "achieved": round(sec_gbs, 1), "peak": HBM_PEAK_GBS,
                  "unit": "GB/s", "frac": round(sec_gbs / HBM_PEAK_GBS, 4),
                  "traffic": read_traffic(wl.name, bits, "thc_aggregate_decode") if not a.sat else None}

    dom_ops = (path.size * (path.l + 2.0) if a.full_rotation
               else coords_per_launch * (W if path.fused else 1) * ENCODE_OPS_PER_COORD)
    alu_achieved = dom_ops / dom_s / 1e12
    copy_gbs = copy_bandwidth(torch, dev)

    sb = path.sum_bytes
    # the aggregate that an all-reduce would deliver is written once and read once: u8/u16
    # sums for the exact path, b bits for the saturating one
    agg_bytes = bits / 8.0 if a.sat else sb
    alg_bytes_per_coord = W * (s_in + bits / 8.0) + W * bits / 8.0 + 2 * agg_bytes + 4
    moved_bytes_per_coord = alg_bytes_per_coord - (2 * agg_bytes if (path.fused and path.no_sums) else 0)
    if a.full_rotation:
        moved_bytes_per_coord = alg_bytes_per_coord
    value = W * wl.n * s_in / (ms * 1e-3) / 1e9
    res = {
        "metric": "gradient GB/s for encode+aggregate+decode (W workers) and % of HBM peak, 1 GPU",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": W, "n": wl.n, "input": wl.dtype, "bits": bits,
                   "chunk_log2": wl.chunk_log2, "buckets": nb, "bucket_elems": wl.bucket or wl.n,
                   "form": "fused" if path.fused else "unfused",
                   "launches": "one thc_encode_all_cleared + one thc_aggregate_decode per bucket"
                               if path.fused else "one call per step of the method",
                   "aggregation": "saturating" if a.sat else "exact",
                   "rotation": f"full, 2^{path.l}" if a.full_rotation else "partial",
                   "philox_seed": 0 if a.full_rotation else "bucket index (0 .. buckets - 1)",
                   "data_seed": "1000 * configuration + worker"},
        "step_time_ms": {"statistic": "median of per-step HIP-event pairs", "median": round(ms, 4),
                         "mean": round(ms_mean, 4), "min": round(ms_min, 4), "max": round(ms_max, 4)},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": read_traffic(wl.name, bits, dom_name)},
        "roofline_alu": {"bound": "alu", "kernel": dom_name, "achieved": round(alu_achieved, 2),
                         "peak": round(VALU_PEAK_TOPS, 2), "unit": "Top/s",
                         "frac": round(alu_achieved / VALU_PEAK_TOPS, 4),
                         "ops_per_worker_coord": ENCODE_OPS_PER_COORD,
                         "ops_per_worker_coord_executed": read_executed_ops(wl.name, bits) if path.fused and not a.sat
                         and not a.full_rotation else None},
        "roofline_second": second,
        "pct_hbm_peak": round(100.0 * wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "copy_GBps": round(copy_gbs, 1),
        "pipeline_hbm": {"algorithmic_bytes_per_coord": alg_bytes_per_coord,
                         "achieved_GBps": round(wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "frac_of_copy": round(wl.n * alg_bytes_per_coord / (ms * 1e-3) / 1e9 / copy_gbs, 4),
                         # what the timed calls really move: the fused decoder never stores the sums
                         "moved_bytes_per_coord": moved_bytes_per_coord,
                         "moved_GBps": round(wl.n * moved_bytes_per_coord / (ms * 1e-3) / 1e9, 1),
                         "moved_frac_of_peak": round(wl.n * moved_bytes_per_coord / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "kernels": kernels,
    }
    # by the traffic counters: bytes the two kernels were measured to move per launch of the
    # first bucket (rocprofv3, committed under profiles/), per coordinate of that bucket
    t_enc = read_traffic(wl.name, bits, "thc_encode_all")
    t_dec = read_traffic(wl.name, bits, "thc_aggregate_decode")
    if path.fused and not a.sat and not a.full_rotation and t_enc and t_dec:
        per_coord = (t_enc + t_dec) / float(path.items[0]["ln"])
        res["pipeline_hbm"]["counter_bytes_per_coord"] = round(per_coord, 3)
        res["pipeline_hbm"]["counter_frac_of_peak"] = round(wl.n * per_coord / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if a.full_rotation:
        path.step()   # the per-kernel loops above left scratch in the buffers: one clean pass
        torch.cuda.synchronize()
        mean = torch.zeros(wl.n, dtype=torch.float32, device=dev)
        for x in xs:
            mean += x.float()
        mean /= W
        res["vnmse"] = float(((path.out - mean) ** 2).sum() / (mean ** 2).sum())
    if path.fused and not a.sat:
        res["vnmse_first_bucket"] = vnmse(torch, path, path.items[0])
    if path.fused and not a.sat and not a.full_rotation and nb > 1 and wl.chunk_log2 == 14 and path.no_sums:
        try:
            # the same step through the batched entry points: every bucket in one call of each
            # kind (outputs are byte-identical; reported beside the per-bucket form, which stays
            # the headline because it is the form a bucket-at-a-time caller uses)
            bk = [dict(grads=it["grads"], payloads=it["payloads"], scale=it["scale"], out=it["out"],
                       n=it["ln"], seed=it["seed"]) for it in path.items]
            wsb = torch.empty(thc.thc_batch_workspace_bytes([it["ln"] for it in path.items], W, wl.chunk_log2),
                              dtype=torch.uint8, device=dev)
            ref_out = path.items[-1]["out"].clone()

            def batched():
                thc.thc_encode_all_batch(bk, wl.chunk_log2, bits, wsb)
                thc.thc_aggregate_decode_batch(bk, wl.chunk_log2, bits, wsb)
            batched()
            torch.cuda.synchronize()
            assert not thc.thc_encode_all_timed_out(wsb) and torch.equal(ref_out, path.items[-1]["out"])
            b_med, b_mean, b_min, b_max = time_steps(torch, batched, max(3, a.steps // 2))
            enc_b = time_steps(torch, lambda: thc.thc_encode_all_batch(bk, wl.chunk_log2, bits, wsb), 5)[0]
            dec_b = time_steps(torch, lambda: thc.thc_aggregate_decode_batch(bk, wl.chunk_log2, bits, wsb), 5)[0]
            res["batched"] = {"form": "thc_encode_all_batch + thc_aggregate_decode_batch, all buckets per call",
                              "ms_per_step": round(b_med, 4), "value": round(W * wl.n * s_in / (b_med * 1e-3) / 1e9, 2),
                              "pct_hbm_peak": round(100.0 * wl.n * alg_bytes_per_coord / (b_med * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
                              "encode_ms_per_step": round(enc_b, 4), "decode_ms_per_step": round(dec_b, 4)}
        except Exception as e:   # a side measurement: report, do not lose the headline
            res["batched"] = {"error": f"{type(e).__name__}: {e}"}
    if a.sat:
        # quality of the variant on the first bucket, next to the exact-sum path's
        it = path.items[0]
        path.overflow.zero_()
        path.count_overflow = True
        path.encode_all(it)
        path.aggregate_decode(it)
        torch.cuda.synchronize()
        res["sat"] = {"overflow_rate": round(int(path.overflow.item()) / it["ln"], 6),
                      "vnmse": vnmse(torch, path, it)}
        ref = dict(it, out=torch.empty_like(it["out"]), scale=torch.empty_like(it["scale"]),
                   payloads=[torch.empty_like(p) for p in it["payloads"]],
                   sums=torch.empty(it["P"] << path.l, dtype=torch.uint8 if sb == 1 else torch.int16,
                                    device=dev))
        thc.thc_encode_all(ref["grads"], path.l, ref["seed"], bits, ref["payloads"], ref["scale"], ref["ws"])
        thc.thc_aggregate_decode(ref["payloads"], ref["scale"], ref["ln"], path.l, ref["seed"], bits,
                                 ref["sums"], ref["out"])
        torch.cuda.synchronize()
        res["sat"]["vnmse_exact_sums"] = vnmse(torch, path, ref)
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, bits, xs, a.cpu_sample_log2)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
