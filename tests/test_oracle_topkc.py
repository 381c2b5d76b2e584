"""Pins for the TopKC oracle (CPU only): exact small-integer cases, brute-force selection,
the library's fp16 conversion and addition, the paper's cost formula, and the qualitative
claims the paper makes about the method."""
import numpy as np
import pytest
import torch

from oracle.topkc import (bits_per_coordinate, chunk_norms, gather_sum, num_chunks, pipeline,
                          scatter_mean, select, sum_fp16)


def test_cost_formula_values():
    # b = 16 (J C / d + 1 / C)
    assert bits_per_coordinate(J=1000, C=64, d=6_400_000) == pytest.approx(16 * (0.01 + 1 / 64))
    assert bits_per_coordinate(J=0, C=128, d=10**9) == pytest.approx(0.125)


def test_norms_exact_on_small_integers():
    """Small integers: every square and partial sum is exact in fp32 and fp16, so the
    result is the mathematical squared norm whatever the summation order."""
    C = 8
    x = np.array([1, 2, 3, 0, -1, 2, 0, 1,   0, 0, 0, 0, 0, 0, 0, 0,   4, -4, 4, -4, 1, 1, 1, 1,   3], dtype=np.float32)
    got = chunk_norms(x, C)
    assert got.dtype == np.float16
    assert got.tolist() == [20.0, 0.0, 68.0, 9.0]            # last chunk zero-padded
    assert num_chunks(len(x), C) == 4


def test_norm_summation_is_the_adjacent_pair_tree_in_fp32():
    """Values chosen so that fp32 summation order matters: the tree order gives a result
    different from left-to-right, and the oracle must give the tree's."""
    C = 4
    x = np.array([4096.0, 1.0 / 64, 1.0 / 64, 1.0 / 64], dtype=np.float32)   # squares: 2^24, 2^-12 x3
    sq = (x * x).astype(np.float32)
    tree = np.float32(np.float32(sq[0] + sq[1]) + np.float32(sq[2] + sq[3]))
    left = np.float32(np.float32(np.float32(sq[0] + sq[1]) + sq[2]) + sq[3])
    assert tree == left            # both lose the tiny terms here; sanity of the construction
    x2 = np.array([1.0, 2.0 ** -12, 2.0 ** -12, 2.0 ** -12] , dtype=np.float32)  # squares 1, 2^-24 x3
    sq = (x2 * x2).astype(np.float32)
    tree = np.float32(np.float32(sq[0] + sq[1]) + np.float32(sq[2] + sq[3]))      # 1 + 2^-23 (pair survives)
    left = np.float32(np.float32(np.float32(sq[0] + sq[1]) + sq[2]) + sq[3])      # 1 (each tiny term rounds away)
    assert tree != left
    # fp16 would hide the difference, so check the fp32 stage through a norm above fp16's ulp:
    big = np.concatenate([x2 * 2.0 ** 6] * 1)                                     # scale by 64: squares x 4096
    got = chunk_norms(big.astype(np.float32), C)
    assert got[0] == np.float16(np.float32(tree) * np.float32(4096.0))


def test_fp16_rounding_and_addition_match_the_library():
    rng = np.random.default_rng(0)
    a = (rng.normal(size=50_000) * 10.0 ** rng.integers(-8, 4, size=50_000)).astype(np.float32)
    b = (rng.normal(size=50_000) * 10.0 ** rng.integers(-8, 4, size=50_000)).astype(np.float32)
    ha, hb = a.astype(np.float16), b.astype(np.float16)
    assert (ha.view(np.uint16) == torch.from_numpy(a).to(torch.float16).view(torch.int16).numpy().view(np.uint16)).all()
    want = (torch.from_numpy(ha) + torch.from_numpy(hb)).numpy()
    got = sum_fp16([ha, hb])
    assert (got.view(np.uint16) == want.view(np.uint16)).all()


def test_sum_is_in_worker_order():
    """fp16 addition is not associative: 2048 + 1 + 1 is 2048 left to right (each 1 is half
    an ulp and ties to even) but 2050 if the ones are added first."""
    a = [np.array([2048.0], dtype=np.float16), np.array([1.0], dtype=np.float16), np.array([1.0], dtype=np.float16)]
    assert sum_fp16(a)[0] == 2048.0
    assert sum_fp16(a[::-1])[0] == 2050.0


def test_select_brute_force_with_ties():
    rng = np.random.default_rng(1)
    for trial in range(20):
        P = int(rng.integers(5, 300))
        s = rng.integers(0, 6, size=P).astype(np.float16)       # many ties
        J = int(rng.integers(1, P + 1))
        got = select(s, J)
        # brute force: repeatedly take the largest value, lowest index first
        taken, left = [], list(range(P))
        for _ in range(J):
            best = max(left, key=lambda i: (float(s[i]), -i))
            taken.append(best)
            left.remove(best)
        assert got.tolist() == sorted(taken)
        assert (np.diff(got.astype(np.int64)) > 0).all()


def test_select_handles_inf_and_subnormals():
    s = np.array([0.0, np.inf, 6e-8, 65504.0, 6e-8, 0.0], dtype=np.float16)
    assert select(s, 1).tolist() == [1]
    assert select(s, 3).tolist() == [1, 2, 3]
    assert select(s, 4).tolist() == [1, 2, 3, 4]
    assert select(s, 5).tolist() == [0, 1, 2, 3, 4]


def test_gather_scatter_exact_on_small_integers():
    C, W = 4, 3
    xs = [np.arange(12, dtype=np.float32) * (w + 1) for w in range(W)]     # chunk p of worker w: (w+1) * [4p..4p+3]
    vals = gather_sum(xs, C, [0, 2])
    assert vals.dtype == np.float16
    assert vals.tolist() == [[0.0, 6.0, 12.0, 18.0], [48.0, 54.0, 60.0, 66.0]]
    out = scatter_mean(vals, [0, 2], C, W, 11)
    assert out.tolist() == [0.0, 2.0, 4.0, 6.0, 0, 0, 0, 0, 16.0, 18.0, 20.0]


def test_all_chunks_selected_is_the_fp16_dense_sum():
    rng = np.random.default_rng(2)
    C, W, d = 16, 4, 1000
    xs = [rng.normal(size=d).astype(np.float32) for _ in range(W)]
    res = pipeline(xs, C, num_chunks(d, C))
    dense = sum_fp16([x.astype(np.float16) for x in xs]).astype(np.float32) / np.float32(W)
    assert (res["out"] == dense).all()
    assert res["indices"].tolist() == list(range(num_chunks(d, C)))


def test_error_falls_as_more_chunks_are_sent_and_locality_helps():
    """vNMSE decreases with J, and shuffling the coordinates (no spatial locality) makes
    TopKC worse at the same J: the comparison the paper uses to justify chunks."""
    rng = np.random.default_rng(3)
    C, W, d = 64, 4, 1 << 16
    layer_scale = np.repeat(10.0 ** rng.uniform(-3, 0, size=d // 1024), 1024)      # large values cluster
    xs = [(rng.normal(size=d) * layer_scale).astype(np.float32) for _ in range(W)]
    mean = np.mean(xs, axis=0, dtype=np.float64)
    errs = []
    for J in (8, 64, 256, 1024):
        out = pipeline(xs, C, J)["out"]
        errs.append(np.sum((out - mean) ** 2) / np.sum(mean ** 2))
    assert errs[0] > errs[1] > errs[2] > errs[3]
    perm = rng.permutation(d)
    xp = [x[perm] for x in xs]
    out_p = pipeline(xp, C, 256)["out"]
    err_p = np.sum((out_p - mean[perm]) ** 2) / np.sum(mean ** 2)
    assert err_p > 1.5 * errs[2]
