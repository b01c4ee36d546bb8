"""Pins of the oracle's non-negative factorisation (Algorithm 1's first step, Sec. 2.1; the paper uses a library and
names no algorithm, so these pin the algorithm chosen, Lee and Seung's multiplicative updates, to the mathematics)."""
import numpy as np
import pytest

from oracle import nmf


def test_objective_never_increases_and_factors_stay_non_negative():
    rng = np.random.default_rng(0)
    for (r, c, k) in [(5, 5, 2), (20, 30, 4), (64, 48, 8)]:
        M = np.abs(rng.normal(size=(r, c)))
        hist = []
        Mp, Mz = nmf.nmf_tile(M, rng.random((r, k)), rng.random((k, c)), 40, history=hist)
        assert all(b <= a * (1 + 1e-12) for a, b in zip(hist, hist[1:])), "Lee and Seung: monotone"
        assert hist[-1] < 0.9 * hist[0]
        assert (Mp >= 0).all() and (Mz >= 0).all()


def test_exact_factorisation_is_a_fixed_point():
    rng = np.random.default_rng(1)
    A, B = rng.random((12, 3)) + 0.1, rng.random((3, 9)) + 0.1
    Mp, Mz = nmf.nmf_tile(A @ B, A, B, 5, eps=1e-12)
    assert np.allclose(Mp, A, rtol=1e-9) and np.allclose(Mz, B, rtol=1e-9)


def test_rank_one_update_is_the_least_squares_solution():
    """k = 1: M_z <- M_z (M_p^T M) / (M_p^T M_p M_z) = M_p^T M / |M_p|^2, the least-squares row for the given column."""
    rng = np.random.default_rng(2)
    M = np.abs(rng.normal(size=(7, 6)))
    p0, z0 = rng.random((7, 1)) + 0.1, rng.random((1, 6)) + 0.1
    z1 = z0 * (p0.T @ M) / (p0.T @ p0 @ z0 + 0.0)
    assert np.allclose(z1, np.linalg.lstsq(p0, M, rcond=None)[0])
    # and the oracle's first half-step is exactly that
    Mp, Mz = nmf.nmf_tile(M, p0, z0, 1, eps=0.0)
    p1 = np.linalg.lstsq(z1.T, M.T, rcond=None)[0].T
    assert np.allclose(Mz, z1) and np.allclose(Mp, p1)


def test_manipulation_methods_on_a_handwritten_matrix():
    # Sec. 3.2: manipulation acts elementwise on the magnitudes before the factorisation (values worked out by hand)
    W = np.array([[-0.1, 0.9, -1.2], [1.4, -0.2, 0.8]])
    assert np.array_equal(nmf.magnitude(W, 1), np.abs(W))
    assert np.allclose(nmf.magnitude(W, 2), W * W)
    m3 = nmf.magnitude(W, 3, w_threshold=0.8, S=0.5)
    assert np.allclose(m3, [[0.1, 1.8, 2.4], [2.8, 0.2, 1.6]])      # >= threshold doubled (1 / (1 - 0.5)), the rest kept
    with pytest.raises(ValueError):
        nmf.magnitude(W, 4)


def test_tiles_are_independent_and_cut_off_tiles_are_smaller_tiles():
    rng = np.random.default_rng(3)
    m, n, r, c, k = 11, 14, 4, 5, 2
    T = 3 * 3
    W = rng.normal(size=(m, n))
    Mp0, Mz0 = rng.random((T, r, k)), rng.random((T, k, c))
    Mp, Mz = nmf.nmf(W, Mp0, Mz0, r, c, 7)
    for t in range(T):
        ti, tj = divmod(t, 3)
        Wt = np.abs(W[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c])
        rt, ct = Wt.shape
        p, z = nmf.nmf_tile(Wt, Mp0[t, :rt], Mz0[t, :, :ct], 7)
        assert np.array_equal(Mp[t, :rt], p) and np.array_equal(Mz[t, :, :ct], z)
        assert np.array_equal(Mp[t, rt:], Mp0[t, rt:]) and np.array_equal(Mz[t, :, ct:], Mz0[t, :, ct:])
