"""CPU oracle for the non-negative factorisation step of Algorithm 1 (arXiv 1905.05686, Sec. 2.1), tile by tile.

TEST INFRASTRUCTURE ONLY: plain numpy in float64, one tile at a time.  Shares no code with the GPU library.

The paper factorises the magnitude matrix M = |W| into non-negative M_p (r x k) and M_z (k x c) that minimise the
Frobenius distance |M - M_p M_z|_F^2 with an off-the-shelf library and does not name the algorithm.  Reading taken
here (the same one the library's header states): the multiplicative updates of Lee and Seung for the Frobenius
objective, from a starting point the caller provides (the random numbers are inputs), M_z first, then M_p, `iters`
times:
    M_z <- M_z * (M_p^T M) / (M_p^T M_p M_z + eps)
    M_p <- M_p * (M M_z^T) / (M_p M_z M_z^T + eps)        (products elementwise, eps > 0 guards 0 / 0)
Because the library is unspecified, factors are comparable with the paper's only statistically: PARITY UNPINNED by
the paper's numbers; the pins below fix the algorithm itself.

Weight-magnitude manipulation (Sec. 3.2) acts on M before the factorisation:
    method 1: M = |W|;  method 2: M = |W|^2;  method 3: M = |W| / (1 - S) where |W| >= w_threshold, |W| elsewhere
(S the sparsity of magnitude pruning; "larger than a threshold" is read as the kept set of Eq. 1 -> Eq. 2, >=).
A tile cut off at the matrix edge is factorised as the smaller tile it is; the unused rows / columns of its factors
are left as given.
Pins: tests/test_oracle_nmf.py (the objective never increases: Lee and Seung's theorem; an exact non-negative
factorisation is a fixed point; with k = 1 one update is the least-squares solution, checked against numpy.linalg;
non-negativity; tiles are independent; the manipulation methods on the printed 5 x 5 example).
"""
import numpy as np


def magnitude(W, method=1, w_threshold=0.0, S=0.0):
    A = np.abs(np.asarray(W, dtype=np.float64))
    if method == 1:
        return A
    if method == 2:
        return A * A
    if method == 3:
        return np.where(A >= w_threshold, A * (1.0 / (1.0 - S)), A)
    raise ValueError("method must be 1, 2 or 3")


def objective(M, Mp, Mz):
    D = M - Mp @ Mz
    return float((D * D).sum())


def nmf_tile(M, Mp, Mz, iters, eps=1e-9, history=None):
    """Multiplicative updates on one tile; returns the updated (Mp, Mz).  `history`, if a list, receives the
    objective before the first and after every iteration."""
    M = np.asarray(M, dtype=np.float64)
    Mp = np.array(Mp, dtype=np.float64)
    Mz = np.array(Mz, dtype=np.float64)
    if history is not None:
        history.append(objective(M, Mp, Mz))
    for _ in range(iters):
        Mz = Mz * (Mp.T @ M) / (Mp.T @ Mp @ Mz + eps)
        Mp = Mp * (M @ Mz.T) / (Mp @ (Mz @ Mz.T) + eps)
        if history is not None:
            history.append(objective(M, Mp, Mz))
    return Mp, Mz


def nmf(W, Mp0, Mz0, r, c, iters, eps=1e-9, method=1, w_threshold=0.0, S=0.0):
    """All tiles of a layer.  W [m, n]; Mp0 [T, r, k], Mz0 [T, k, c] starting points.  Returns float64 factors."""
    A = magnitude(W, method, w_threshold, S)
    m, n = A.shape
    tile_cols = -(-n // c)
    T = -(-m // r) * tile_cols
    Mp = np.array(Mp0, dtype=np.float64)
    Mz = np.array(Mz0, dtype=np.float64)
    if Mp.shape[0] != T or Mz.shape[0] != T:
        raise ValueError("one pair of factors per tile")
    for t in range(T):
        ti, tj = divmod(t, tile_cols)
        Mt = A[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c]
        rt, ct = Mt.shape
        p, z = nmf_tile(Mt, Mp[t, :rt, :], Mz[t, :, :ct], iters, eps)
        Mp[t, :rt, :] = p
        Mz[t, :, :ct] = z
    return Mp, Mz
