"""Pins for the oracle's rotation: explicit Hadamard matrices, closed forms,
invariants (CPU only)."""
import numpy as np
import pytest
import scipy.linalg

from oracle.thc import fwht, num_chunks, rht_forward, rht_inverse, sign_bits

H2 = np.array([[1, 1],
               [1, -1]], dtype=np.float64)
H4 = np.array([[1, 1, 1, 1],
               [1, -1, 1, -1],
               [1, 1, -1, -1],
               [1, -1, -1, 1]], dtype=np.float64)
H8 = np.array([[1, 1, 1, 1, 1, 1, 1, 1],
               [1, -1, 1, -1, 1, -1, 1, -1],
               [1, 1, -1, -1, 1, 1, -1, -1],
               [1, -1, -1, 1, 1, -1, -1, 1],
               [1, 1, 1, 1, -1, -1, -1, -1],
               [1, -1, 1, -1, -1, 1, -1, 1],
               [1, 1, -1, -1, -1, -1, 1, 1],
               [1, -1, -1, 1, -1, 1, 1, -1]], dtype=np.float64)


def _matrix_of(c, dtype=np.float64):
    """Columns = fwht(e_k)."""
    return fwht(np.eye(c, dtype=dtype)).T.copy()


@pytest.mark.parametrize("H", [H2, H4, H8])
def test_small_hadamard_matrices(H):
    c = len(H)
    assert (_matrix_of(c) == H).all()
    assert (_matrix_of(c, np.float32) == H).all()
    # the literal matrices themselves follow the Sylvester recursion
    if c > 2:
        h = H[:c // 2, :c // 2]
        assert (H == np.block([[h, h], [h, -h]])).all()


@pytest.mark.parametrize("log2c", [1, 4, 7, 10])
def test_matches_scipy_and_popcount_closed_form(log2c):
    c = 1 << log2c
    M = _matrix_of(c)
    assert (M == scipy.linalg.hadamard(c)).all()
    i = np.arange(c)
    pc = np.array([[bin(a & b).count("1") for b in i] for a in i]) if c <= 128 else None
    if pc is not None:
        assert (M == (-1.0) ** pc).all()
    assert (M @ M == c * np.eye(c)).all()


def test_constant_vector_becomes_a_spike():
    c = 64
    a = fwht(np.full((1, c), 0.25))
    want = np.zeros(c)
    want[0] = 0.25 * c
    assert (a[0] == want).all()


def test_delta_spreads_to_a_column():
    c = 32
    for k in (0, 5, 31):
        e = np.zeros((1, c))
        e[0, k] = 1.0
        assert (fwht(e)[0] == scipy.linalg.hadamard(c)[:, k]).all()


@pytest.mark.parametrize("log2c,P", [(2, 3), (3, 2), (5, 4)])
def test_partial_rotation_is_block_diagonal(log2c, P):
    """l' stages = kron(I_P, H_c / sqrt(c)) applied to D x."""
    c = 1 << log2c
    rng = np.random.default_rng(log2c)
    x = rng.standard_normal(P * c).astype(np.float32)
    seed = 99
    D = np.where(sign_bits(0, P * c, seed), -1.0, 1.0)
    big = np.kron(np.eye(P), scipy.linalg.hadamard(c) / np.sqrt(c))
    want = big @ (D * x.astype(np.float64))
    got = rht_forward(x, log2c, seed)
    assert np.allclose(got, want, rtol=0, atol=1e-13)
    got32 = rht_forward(x, log2c, seed, dtype=np.float32)
    assert got32.dtype == np.float32
    assert np.allclose(got32, want, rtol=0, atol=2e-6)
    # and the inverse is the transpose of an orthogonal matrix
    back = rht_inverse(got, P * c, log2c, seed)
    assert np.allclose(back, x, rtol=0, atol=1e-13)
    assert np.allclose(D * (big.T @ got), x, atol=1e-13)


@pytest.mark.parametrize("log2c", [1, 3, 10, 14])
def test_parseval_and_round_trip(log2c):
    c = 1 << log2c
    rng = np.random.default_rng(3)
    n = 3 * c
    x = (rng.standard_t(3, size=n) * 1e-3).astype(np.float32)
    y = rht_forward(x, log2c, 17)
    ny = np.linalg.norm(y.reshape(3, c), axis=1)
    nx = np.linalg.norm(x.astype(np.float64).reshape(3, c), axis=1)
    assert np.allclose(ny, nx, rtol=1e-12)
    assert np.allclose(rht_inverse(y, n, log2c, 17), x, rtol=0, atol=1e-15)
    y32 = rht_forward(x, log2c, 17, dtype=np.float32)
    ny32 = np.linalg.norm(y32.astype(np.float64).reshape(3, c), axis=1)
    assert np.allclose(ny32, nx, rtol=1e-6)
    x32 = rht_inverse(y32, n, log2c, 17, dtype=np.float32)
    assert np.linalg.norm(x32 - x) <= 1e-6 * np.linalg.norm(x)
    assert np.linalg.norm(y32 - y) <= 1e-6 * np.linalg.norm(y)


def test_chunks_are_independent():
    log2c, P = 6, 5
    c = 1 << log2c
    rng = np.random.default_rng(0)
    x = rng.standard_normal(P * c).astype(np.float32)
    y = rht_forward(x, log2c, 1)
    x2 = x.copy()
    x2[2 * c + 7] += 1.0
    y2 = rht_forward(x2, log2c, 1)
    changed = (y != y2).reshape(P, c).any(axis=1)
    assert changed.tolist() == [False, False, True, False, False]
    # every coordinate of the touched chunk moves by exactly 1/sqrt(c) in magnitude
    assert np.allclose(np.abs(y2 - y).reshape(P, c)[2], 1 / np.sqrt(c))


def test_same_diagonal_for_all_workers_so_rotation_commutes_with_the_sum():
    log2c = 8
    rng = np.random.default_rng(1)
    xs = [rng.standard_normal(1000).astype(np.float32) for _ in range(4)]
    ys = [rht_forward(x, log2c, 5) for x in xs]
    tot = rht_forward(np.sum([x.astype(np.float64) for x in xs], axis=0), log2c, 5)
    assert np.allclose(np.sum(ys, axis=0), tot, atol=1e-12)


def test_signs_are_applied_before_the_transform_and_undone_after():
    # D e_k = -e_k where the bit is set: forward of e_k is +-column k
    log2c, seed = 4, 3
    c = 1 << log2c
    neg = sign_bits(0, c, seed)
    assert neg.any() and (~neg).any()
    H = scipy.linalg.hadamard(c) / np.sqrt(c)
    for k in range(c):
        e = np.zeros(c, dtype=np.float32)
        e[k] = 1.0
        want = -H[:, k] if neg[k] else H[:, k]
        assert np.allclose(rht_forward(e, log2c, seed), want, atol=1e-15)
        # inverse applies D last: H e_k then D
        want_inv = np.where(neg, -1.0, 1.0) * H[:, k]
        assert np.allclose(rht_inverse(e, c, log2c, seed), want_inv, atol=1e-15)


def test_ragged_tail_is_zero_padding_and_is_dropped_again():
    log2c = 5
    c = 32
    rng = np.random.default_rng(2)
    n = 3 * c + 11
    x = rng.standard_normal(n).astype(np.float32)
    assert num_chunks(n, log2c) == 4
    xp = np.zeros(4 * c, dtype=np.float32)
    xp[:n] = x
    y = rht_forward(x, log2c, 8)
    assert y.shape == (4 * c,)
    assert (y == rht_forward(xp, log2c, 8)).all()
    back = rht_inverse(y, n, log2c, 8)
    assert back.shape == (n,)
    assert np.allclose(back, x, atol=1e-14)


def test_window_with_global_offset_matches_whole():
    log2c = 6
    c = 64
    rng = np.random.default_rng(4)
    x = rng.standard_normal(5 * c).astype(np.float32)
    y = rht_forward(x, log2c, 21).reshape(5, c)
    y3 = rht_forward(x[3 * c:4 * c], log2c, 21, g0=3 * c)
    assert (y3 == y[3]).all()
    assert (rht_inverse(y[3], c, log2c, 21, g0=3 * c) == rht_inverse(y.reshape(-1), 5 * c, log2c, 21)[3 * c:4 * c]).all()


def test_bf16_patterns_are_widened_exactly():
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x4049, 0x3DCD], dtype=np.uint16)  # 1, -1, 0, 3.140625, 0.10009765625
    # seed whose first 8 sign bits we undo by hand
    seed = 0
    neg = sign_bits(0, 8, seed)
    y = rht_forward(bits, 3, seed, bf16=True)
    vals = np.array([1.0, -1.0, 0.0, 3.140625, 0.10009765625, 0, 0, 0])
    vals = np.where(neg, -vals, vals)
    assert np.allclose(y, scipy.linalg.hadamard(8) @ vals / np.sqrt(8), atol=1e-15)


def test_rotation_makes_heavy_tails_look_normal():
    """After the rotation the entries are close to zero-mean normal (the paper's
    motivation for saturation): excess kurtosis of a Student-t(3) chunk vanishes."""
    rng = np.random.default_rng(6)
    x = rng.standard_t(3, size=1 << 14).astype(np.float32)
    y = rht_forward(x, 14, 2)
    k_in = ((x - x.mean()) ** 4).mean() / x.var() ** 2
    k_out = ((y - y.mean()) ** 4).mean() / y.var() ** 2
    assert k_in > 6
    assert abs(k_out - 3) < 0.3
    assert np.abs(y).max() < np.abs(x).max()


def test_full_rotation_splits_into_chunk_stages_then_a_small_hadamard_across_chunks():
    """H_(2^17) = H_8 (x) H_(2^14): the 17 stages of a full rotation are the 14 stages inside
    every 2^14 chunk followed by an 8-point Hadamard matrix (closed form) across the 8
    chunks.  Pins the oracle's stage structure above the largest chunk size."""
    rng = np.random.default_rng(17)
    x = rng.normal(size=1 << 17)
    full = fwht(x.copy())
    per_chunk = fwht(x.copy().reshape(8, 1 << 14))              # stages 0..13, chunk by chunk
    H8 = np.array([[(-1) ** bin(i & j).count("1") for j in range(8)] for i in range(8)], dtype=np.float64)
    want = (H8 @ per_chunk).reshape(-1)
    assert np.allclose(full, want, rtol=0, atol=1e-9 * np.abs(want).max())


def test_full_rotation_through_the_public_functions_is_an_isometry_and_inverts():
    rng = np.random.default_rng(5)
    n, l = 100_000, 17
    x = rng.normal(size=n).astype(np.float32)
    y = rht_forward(x, l, 3)
    assert y.size == 1 << l
    assert abs(np.linalg.norm(y) - np.linalg.norm(x.astype(np.float64))) < 1e-9 * np.linalg.norm(x)
    assert np.allclose(rht_inverse(y, n, l, 3), x, rtol=0, atol=1e-12)
