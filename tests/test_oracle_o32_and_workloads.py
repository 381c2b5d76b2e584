"""The float32 canonical-order oracle is pinned by the float64 definition, and
the whole path runs on inputs shaped like the named workloads (CPU only)."""
import numpy as np
import pytest

from oracle import thc as O
from synth import generate, to_numpy_bits, workload


def _band(t64):
    """True where the float64 pre-rounding value is within 1e-6 relative of a
    grid boundary (an integer of t): the only place indices may differ."""
    return np.abs(t64 - np.rint(t64)) <= 1e-6 * np.maximum(1.0, np.abs(t64))


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("log2c", [10, 14])
def test_float32_path_agrees_with_float64_definition(bits, log2c):
    rng = np.random.default_rng(bits * 100 + log2c)
    W = 3
    n = (1 << log2c) * 2 + 1234
    xs = [(rng.standard_t(3, size=n) * 10.0 ** rng.uniform(-5, -2)).astype(np.float32) for _ in range(W)]
    o64 = O.pipeline(xs, log2c, 7, bits, dtype=np.float64)
    o32 = O.pipeline(xs, log2c, 7, bits, dtype=np.float32)
    for w in range(W):
        assert o32["y"][w].dtype == np.float32
        ny = np.linalg.norm(o64["y"][w])
        assert np.linalg.norm(o32["y"][w] - o64["y"][w]) <= 1e-6 * ny
        diff = o32["idx"][w] != o64["idx"][w]
        # the float32 path's own t may differ from the float64 t by float32 rounding of
        # v (about L * 2^-23): indices may only differ where float64 t is that close
        # to an integer
        L = (1 << bits) - 1
        slack = np.abs(o64["t"][w] - np.rint(o64["t"][w])) <= 4 * L * 2.0 ** -23 + 1e-6
        assert (slack | ~diff).all()
        assert diff.mean() < 1e-3
    assert np.allclose(o32["scale"], o64["scale"], rtol=1e-6)
    # stage-wise decode: same sums and scales in, float32 vs float64 arithmetic
    d64 = O.decode(o32["sums"], o32["scale"].astype(np.float64), W, n, log2c, 7, bits, dtype=np.float64)
    d32 = O.decode(o32["sums"], o32["scale"], W, n, log2c, 7, bits, dtype=np.float32)
    assert d32.dtype == np.float32
    assert np.linalg.norm(d32 - d64) <= 1e-5 * np.linalg.norm(d64)


def test_band_helper_is_relative():
    t = np.array([0.0000005, 0.5, 14.99999, 200.0001, 200.001])
    assert _band(t).tolist() == [True, False, True, True, False]


@pytest.mark.parametrize("name,bits", [("tiny", 4), ("resnet50", 4), ("bert_base", 4),
                                        ("gpt_345m", 2), ("gpt_345m", 8), ("gpt_1p3b", 4)])
def test_whole_path_on_workload_shaped_slices(name, bits):
    wl = workload(name)
    assert bits in wl.bits
    W = min(wl.W, 3)
    m = (1 << wl.chunk_log2) * 2 + 333
    xs = [to_numpy_bits(generate(wl, w, "cpu", max_elems=m)) for w in range(W)]
    bf16 = wl.dtype == "bf16"
    assert xs[0].dtype == (np.uint16 if bf16 else np.float32)
    out = O.pipeline(xs, wl.chunk_log2, 0, bits, dtype=np.float32, bf16=bf16)
    L = (1 << bits) - 1
    assert out["sums"].max() <= W * L
    assert out["out"].shape == (m,)
    assert len(out["payloads"][0]) == O.payload_bytes(m, wl.chunk_log2, bits)
    wide = [(x.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if bf16
            else x.astype(np.float64) for x in xs]
    true = np.mean(wide, axis=0)
    if np.linalg.norm(true) > 0:
        c = 1 << wl.chunk_log2
        bound = np.sum((2 * out["scale"].astype(np.float64) / L) ** 2) * c / (4 * W)
        assert np.sum((out["out"] - true) ** 2) < bound


def test_sparse_embedding_rows_make_all_zero_chunks():
    wl = workload("bert_base")
    x = generate(wl, 0, "cpu", max_elems=1 << 18)
    assert x.dtype.is_floating_point and x.numel() == 1 << 18
    rows = x[: (1 << 18) // 768 * 768].view(-1, 768)
    zero_rows = (rows.float().abs().sum(dim=1) == 0).float().mean()
    assert zero_rows > 0.95
    xs = [to_numpy_bits(x)]
    out = O.pipeline(xs, 14, 0, 4, dtype=np.float32, bf16=True)
    assert (out["scale"] == 0).any()
    z = np.repeat(out["scale"] == 0, 1 << 14)
    assert (out["idx"][0][z] == 0).all()
    assert (out["out"][z[: 1 << 18]] == 0).all()


def test_workload_tables():
    sizes = {"tiny": 1 << 20, "resnet50": 25_557_032, "bert_base": 108_412_416,
             "gpt_345m": 353_551_360, "gpt_1p3b": 1_300_000_000}
    chunks = {"tiny": 1024, "resnet50": 1560, "bert_base": 6617, "gpt_345m": 21580, "gpt_1p3b": 79346}
    for name, n in sizes.items():
        wl = workload(name)
        assert wl.n == n and sum(s.size for s in wl.segments) == n
        assert O.num_chunks(n, wl.chunk_log2) == chunks[name]
    b = workload("gpt_1p3b").buckets()
    assert len(b) == 50 and b[0] == (0, 26_214_400) and b[-1][1] == 15_494_400
    assert sum(ln for _, ln in b) == 1_300_000_000
    assert all(st % (1 << 14) == 0 for st, _ in b)
    # same seed, same worker -> same gradient; other worker -> other values, same layer scales
    wl = workload("tiny")
    a, a2, b1 = generate(wl, 0), generate(wl, 0), generate(wl, 1)
    assert (a == a2).all() and not (a == b1).all()
    sa = a.view(16, -1).std(dim=1)
    sb = b1.view(16, -1).std(dim=1)
    assert ((sa / sb - 1).abs() < 0.05).all()
