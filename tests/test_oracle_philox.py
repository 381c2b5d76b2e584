"""Pins for the oracle's Philox4x32-10 (CPU only)."""
import os

import numpy as np

from oracle.philox import philox4x32_10, philox4x32_10_scalar
from oracle.thc import TAG_ROUND, TAG_SIGN, rounding_fields, sign_bits


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    assert len(rows) == 3
    return rows


def test_published_known_answers_scalar(golden_dir):
    for ctr, key, out in _kat(golden_dir):
        assert list(philox4x32_10_scalar(ctr, key)) == out


def test_published_known_answers_vectorised(golden_dir):
    for ctr, key, out in _kat(golden_dir):
        got = philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1])
        assert got.shape == (1, 4) and got.dtype == np.uint32
        assert got[0].tolist() == out


def test_two_implementations_agree():
    rng = np.random.default_rng(7)
    c = rng.integers(0, 2**32, size=(200, 4), dtype=np.uint64)
    for key in [(0, 0), (0xDEADBEEF, 0x12345678), (2**32 - 1, 1)]:
        vec = philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], key[0], key[1])
        for i in range(len(c)):
            assert tuple(int(v) for v in vec[i]) == philox4x32_10_scalar(c[i], key)


def test_bytes_uniform_and_uncorrelated():
    n = 1 << 16
    w = philox4x32_10(np.arange(n), 0, 3, TAG_ROUND, 11, 0)
    b = w.view(np.uint8).reshape(-1).astype(np.float64)
    cnt = np.bincount(b.astype(np.int64), minlength=256)
    exp = b.size / 256
    chi2 = ((cnt - exp) ** 2 / exp).sum()
    # 255 dof: mean 255, sd ~22.6
    assert 150 < chi2 < 380
    x = b - b.mean()
    lag1 = (x[:-1] * x[1:]).mean() / x.var()
    assert abs(lag1) < 5 / np.sqrt(b.size)


def test_sign_bits_indexing_against_scalar_blocks():
    seed = 0x1234_5678_9ABC_DEF0
    g = [0, 1, 31, 32, 127, 128, 129, 4095, 16384 + 77, (1 << 33) + 5]
    for gi in g:
        blk = gi // 128
        words = philox4x32_10_scalar((blk & 0xFFFFFFFF, blk >> 32, 0, TAG_SIGN),
                                     (seed & 0xFFFFFFFF, seed >> 32))
        want = (words[(gi // 32) % 4] >> (gi % 32)) & 1
        assert bool(sign_bits(gi, 1, seed)[0]) == bool(want)
    # a window is the same as its elements one by one
    win = sign_bits(100, 300, seed)
    one = np.array([sign_bits(100 + i, 1, seed)[0] for i in range(300)])
    assert (win == one).all()


def test_sign_bits_balanced_seeded_and_chunk_dependent():
    a = sign_bits(0, 1 << 16, 0)
    assert abs(a.mean() - 0.5) < 4 * 0.5 / np.sqrt(a.size)
    assert (a != sign_bits(0, 1 << 16, 1)).mean() > 0.4
    assert (a[:1024] != a[1024:2048]).mean() > 0.4          # chunks get different signs
    assert (a == sign_bits(0, 1 << 16, 0)).all()


def test_rounding_fields_layout_and_independence():
    seed = 5
    for rbits in (8, 16, 32):
        E = 128 // rbits
        per_word = 32 // rbits
        r = rounding_fields(0, 4 * E, 2, seed, rbits)
        for g in range(4 * E):
            words = philox4x32_10_scalar((g // E, 0, 2, TAG_ROUND), (seed, 0))
            k = g % E
            want = (words[k // per_word] >> (rbits * (k % per_word))) & ((1 << rbits) - 1)
            assert int(r[g]) == want
        # windows are consistent with the whole
        assert (rounding_fields(E + 3, 2 * E, 2, seed, rbits) == r[E + 3:3 * E + 3]).all()
    r0 = rounding_fields(0, 1 << 14, 0, seed)
    r1 = rounding_fields(0, 1 << 14, 1, seed)
    assert r0.max() == 255 and r0.min() == 0
    assert (r0 == r1).mean() < 0.02                               # workers get their own stream
    assert abs(np.corrcoef(r0.astype(float), r1.astype(float))[0, 1]) < 0.05
