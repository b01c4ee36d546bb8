"""Pins of the oracle's backward pass through the masking layer (Sec. 2: with the mask applied as a layer, retraining
updates the kept weights only).  The two functions are pinned to the forward product (itself pinned elsewhere) through
identities that any mistake in them (a transposed operand, a dropped mask, a wrong index) breaks."""
import numpy as np

from oracle import lrbi_oracle as orc


def _case(seed, m, n, N, density=0.3):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(m, n))
    M = (rng.random((m, n)) < density).astype(np.uint8)
    X = rng.normal(size=(n, N))
    dY = rng.normal(size=(m, N))
    return W, M, X, dY


def test_adjoint_identity_against_the_forward_product():
    for seed, (m, n, N) in enumerate([(7, 5, 3), (20, 33, 1), (16, 16, 16), (3, 40, 9)]):
        W, M, X, dY = _case(seed, m, n, N)
        Y = orc.masked_gemm(W, M, X)
        dX = orc.masked_gemm_t(W, M, dY)
        assert dX.shape == (n, N)
        lhs, rhs = float((dY * Y).sum()), float((dX * X).sum())
        assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
        # a one-hot dY picks out a row of the masked matrix: dX[:, 0] = (W o M)[i, :]
        for i in (0, m - 1):
            e = np.zeros((m, 1))
            e[i] = 1.0
            assert np.array_equal(orc.masked_gemm_t(W, M, e)[:, 0], np.where(M[i] == 1, W[i], 0.0))


def test_weight_gradient_is_the_exact_difference_of_the_linear_loss():
    """L(W) = <dY, (W o M) X> is linear in W, so L(W + t e_ij) - L(W) = t dW_ij exactly (up to rounding)."""
    W, M, X, dY = _case(5, 6, 7, 4, density=0.5)
    dW = orc.masked_grad(dY, X, M)
    L0 = float((dY * orc.masked_gemm(W, M, X)).sum())
    for i in range(6):
        for j in range(7):
            Wp = W.copy()
            Wp[i, j] += 1.0
            L1 = float((dY * orc.masked_gemm(Wp, M, X)).sum())
            assert abs((L1 - L0) - dW[i, j]) <= 1e-11
            if M[i, j] == 0:
                assert dW[i, j] == 0.0      # exactly zero, not a small number


def test_against_numpy_dense_products_on_the_masked_matrix():
    W, M, X, dY = _case(9, 31, 45, 6)
    Wm = W * M
    assert np.allclose(orc.masked_gemm_t(W, M, dY), Wm.T @ dY, rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.masked_grad(dY, X, M), (dY @ X.T) * M, rtol=1e-13, atol=1e-13)
    # non-finite values under pruned weights never reach dX
    Wn = W.copy()
    Wn[M == 0] = np.nan
    assert np.array_equal(orc.masked_gemm_t(Wn, M, dY), orc.masked_gemm_t(W, M, dY))
    # a batch of one, given as vectors
    assert orc.masked_gemm_t(W, M, dY[:, 0]).shape == (45, 1)
    assert orc.masked_grad(dY[:, 0], X[:, 0], M).shape == (31, 45)
