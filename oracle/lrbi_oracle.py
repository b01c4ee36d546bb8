"""ctypes front end of the plain-C CPU oracle (oracle/lrbi_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never calls it and it never
imports the GPU package.

All factor / mask arguments are unpacked uint8 arrays holding 0 or 1:
  Ip01 [T, r, k], Iz01 [T, k, c], mask [m, n]; tiles are numbered row-major.
Weights and activations are float64 arrays that hold values already rounded to
the storage dtype of the configuration under test.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lrbi_oracle.c")
_LIB = os.path.join(_HERE, "liblrbi_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP only for the row loop)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, u64, p = ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p
        lib.lrbi_oracle_decode.argtypes = [i64] * 5 + [p, p, p]
        lib.lrbi_oracle_decode.restype = ctypes.c_int
        lib.lrbi_oracle_decode_ranked.argtypes = [i64] * 5 + [p, p, p, p]
        lib.lrbi_oracle_decode_ranked.restype = ctypes.c_int
        lib.lrbi_oracle_index_bits_ranked.argtypes = [i64] * 5 + [p]
        lib.lrbi_oracle_index_bits_ranked.restype = u64
        lib.lrbi_oracle_masked_gemm.argtypes = [i64] * 3 + [p, p, p, p, ctypes.c_int]
        lib.lrbi_oracle_masked_gemm.restype = ctypes.c_int
        lib.lrbi_oracle_masked_gemm_t.argtypes = [i64] * 3 + [p, p, p, p]
        lib.lrbi_oracle_masked_gemm_t.restype = ctypes.c_int
        lib.lrbi_oracle_masked_grad.argtypes = [i64] * 3 + [p, p, p, p]
        lib.lrbi_oracle_masked_grad.restype = ctypes.c_int
        lib.lrbi_oracle_index_bits.argtypes = [i64] * 5
        lib.lrbi_oracle_index_bits.restype = u64
        lib.lrbi_oracle_dense_bits.argtypes = [i64] * 2
        lib.lrbi_oracle_dense_bits.restype = u64
        lib.lrbi_oracle_popcount.argtypes = [i64, i64, p]
        lib.lrbi_oracle_popcount.restype = u64
        lib.lrbi_oracle_csr_bits.argtypes = [u64, i64, ctypes.c_int, ctypes.c_int]
        lib.lrbi_oracle_csr_bits.restype = u64
        lib.lrbi_oracle_threshold.argtypes = [i64] * 4 + [p] * 6
        lib.lrbi_oracle_threshold.restype = ctypes.c_int
        lib.lrbi_oracle_candidate_cost.argtypes = [i64] * 4 + [p, ctypes.c_double, ctypes.c_int, ctypes.c_double, p, p, p]
        lib.lrbi_oracle_candidate_cost.restype = ctypes.c_int
        _lib = lib
    return _lib


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def num_tiles(m: int, n: int, r: int, c: int) -> int:
    return (-(-m // r)) * (-(-n // c))


def decode_mask(Ip01, Iz01, m: int, n: int, r: int, c: int, k: int, tile_rank=None) -> np.ndarray:
    """Eq. 3 per tile (Sec. 3.1): returns the m x n 0/1 mask, 1 = kept.  Tiles that stick out of the
    matrix are cut off at its edge; tile_rank [T] (optional) limits tile t to its first tile_rank[t] ranks."""
    Ip01 = _c(Ip01, np.uint8)
    Iz01 = _c(Iz01, np.uint8)
    T = num_tiles(m, n, r, c)
    if Ip01.shape != (T, r, k) or Iz01.shape != (T, k, c):
        raise ValueError("factor shapes %s %s do not match T=%d r=%d c=%d k=%d"
                         % (Ip01.shape, Iz01.shape, T, r, c, k))
    rank_ptr = None
    if tile_rank is not None:
        tile_rank = _c(tile_rank, np.int32)
        if tile_rank.shape != (T,):
            raise ValueError("tile_rank must have one entry per tile")
        rank_ptr = tile_rank.ctypes.data
    M = np.empty((m, n), dtype=np.uint8)
    rc = _load().lrbi_oracle_decode_ranked(m, n, r, c, k, rank_ptr, Ip01.ctypes.data, Iz01.ctypes.data,
                                           M.ctypes.data)
    if rc != 0:
        raise ValueError("lrbi_oracle_decode failed: %d" % rc)
    return M


def threshold_factors(Mp, Mz, Tp, Tz):
    """Algorithm 1, "convert (M_p, M_z) into (I_p, I_z)" (Sec. 2.1): entry >= threshold -> 1, per tile.
    Mp [T][r][k], Mz [T][k][c] float32; Tp, Tz [T] float32.  Returns (Ip01, Iz01)."""
    Mp = _c(Mp, np.float32)
    Mz = _c(Mz, np.float32)
    Tp = _c(Tp, np.float32)
    Tz = _c(Tz, np.float32)
    T, r, k = Mp.shape
    c = Mz.shape[2]
    if Mz.shape != (T, k, c) or Tp.shape != (T,) or Tz.shape != (T,):
        raise ValueError("shapes do not match")
    Ip01 = np.empty((T, r, k), dtype=np.uint8)
    Iz01 = np.empty((T, k, c), dtype=np.uint8)
    rc = _load().lrbi_oracle_threshold(T, r, c, k, Mp.ctypes.data, Mz.ctypes.data, Tp.ctypes.data,
                                       Tz.ctypes.data, Ip01.ctypes.data, Iz01.ctypes.data)
    if rc != 0:
        raise ValueError("lrbi_oracle_threshold failed: %d" % rc)
    return Ip01, Iz01


def candidate_cost(W, w_threshold: float, M, r: int, c: int, method: int = 1, amplify: float = 1.0):
    """Algorithm 1, the quantities measured for one candidate (Sec. 2.1), per tile: number of ones of
    I_a, and Cost = sum of the magnitudes of the entries with |W| >= w_threshold (I = 1) that I_a prunes; the
    magnitudes are the manipulated ones of Sec. 3.2 (method 1 |W|, 2 |W|^2, 3 amplify |W| on the kept set).
    W float64 m x n (storage-rounded values), M the decoded 0/1 mask.  Returns (kept uint64 [T], cost float64 [T])."""
    W = _c(W, np.float64)
    M = _c(M, np.uint8)
    m, n = W.shape
    if M.shape != (m, n):
        raise ValueError("shapes do not match")
    T = num_tiles(m, n, r, c)
    kept = np.empty(T, dtype=np.uint64)
    cost = np.empty(T, dtype=np.float64)
    rc = _load().lrbi_oracle_candidate_cost(m, n, r, c, W.ctypes.data, float(w_threshold), int(method),
                                            float(amplify), M.ctypes.data, kept.ctypes.data, cost.ctypes.data)
    if rc != 0:
        raise ValueError("lrbi_oracle_candidate_cost failed: %d" % rc)
    return kept, cost


def masked_gemm(W, M, X, threads: int = 1) -> np.ndarray:
    """Y = (W o M) X in float64; pruned weights are skipped (select, not multiply)."""
    W = _c(W, np.float64)
    M = _c(M, np.uint8)
    X = _c(X, np.float64)
    if X.ndim == 1:
        X = X[:, None]
    m, n = W.shape
    if M.shape != (m, n) or X.shape[0] != n:
        raise ValueError("shape mismatch")
    N = X.shape[1]
    Y = np.empty((m, N), dtype=np.float64)
    rc = _load().lrbi_oracle_masked_gemm(m, n, N, W.ctypes.data, M.ctypes.data, X.ctypes.data,
                                         Y.ctypes.data, int(threads))
    if rc != 0:
        raise ValueError("lrbi_oracle_masked_gemm failed: %d" % rc)
    return Y


def masked_gemm_t(W, M, dY) -> np.ndarray:
    """dX = (W o M)^T dY in float64 (Sec. 2: backward pass through the masking layer); pruned weights are skipped."""
    W = _c(W, np.float64)
    M = _c(M, np.uint8)
    dY = _c(dY, np.float64)
    if dY.ndim == 1:
        dY = dY[:, None]
    m, n = W.shape
    if M.shape != (m, n) or dY.shape[0] != m:
        raise ValueError("shape mismatch")
    N = dY.shape[1]
    dX = np.empty((n, N), dtype=np.float64)
    rc = _load().lrbi_oracle_masked_gemm_t(m, n, N, W.ctypes.data, M.ctypes.data, dY.ctypes.data, dX.ctypes.data)
    if rc != 0:
        raise ValueError("lrbi_oracle_masked_gemm_t failed: %d" % rc)
    return dX


def masked_grad(dY, X, M) -> np.ndarray:
    """dW = (dY X^T) o M in float64: the weight gradient of Y = (W o M) X; pruned weights get exactly 0."""
    dY = _c(dY, np.float64)
    X = _c(X, np.float64)
    M = _c(M, np.uint8)
    if dY.ndim == 1:
        dY = dY[:, None]
    if X.ndim == 1:
        X = X[:, None]
    m, n = M.shape
    N = dY.shape[1]
    if dY.shape != (m, N) or X.shape != (n, N):
        raise ValueError("shape mismatch")
    dW = np.empty((m, n), dtype=np.float64)
    rc = _load().lrbi_oracle_masked_grad(m, n, N, dY.ctypes.data, X.ctypes.data, M.ctypes.data, dW.ctypes.data)
    if rc != 0:
        raise ValueError("lrbi_oracle_masked_grad failed: %d" % rc)
    return dW


def index_bits(m: int, n: int, r: int, c: int, k: int, tile_rank=None) -> int:
    """Sum over tiles of k_t (r_t + c_t): Sec. 2.2's k(m+n) applied to every tile of Sec. 3.1
    (tiles * k * (r + c) when the tiles divide the matrix and share one rank)."""
    rank_ptr = None
    if tile_rank is not None:
        tile_rank = _c(tile_rank, np.int32)
        if tile_rank.shape != (num_tiles(m, n, r, c),):
            raise ValueError("tile_rank must have one entry per tile")
        rank_ptr = tile_rank.ctypes.data
    v = int(_load().lrbi_oracle_index_bits_ranked(m, n, r, c, k, rank_ptr))
    if v == 0:
        raise ValueError("invalid shape")
    return v


def dense_bits(m: int, n: int) -> int:
    """One bit per weight (the 'Binary' row of Tables 1 and 3)."""
    return int(_load().lrbi_oracle_dense_bits(m, n))


def compression_ratio(m: int, n: int, r: int, c: int, k: int) -> float:
    """mn / (k(m+n)) of Sec. 2.2, generalised to tiles."""
    return dense_bits(m, n) / index_bits(m, n, r, c, k)


def popcount(M) -> int:
    M = _c(M, np.uint8)
    return int(_load().lrbi_oracle_popcount(M.shape[0], M.shape[1], M.ctypes.data))


def density(M) -> float:
    """Fraction of kept weights, 1 - S_a in the notation of Eq. 7."""
    M = _c(M, np.uint8)
    return popcount(M) / float(M.shape[0] * M.shape[1])


def csr_bits(nnz: int, m: int, idx_bits: int = 16, ptr_bits: int = 32) -> int:
    """Builder's CSR accounting (parity unpinned: the paper prints no formula)."""
    return int(_load().lrbi_oracle_csr_bits(nnz, m, idx_bits, ptr_bits))


def rel_err(y, y_ref) -> float:
    """Error metric of the parity gate: max |y - y_ref| / max(|y_ref|, rms(y_ref)).

    Plain elementwise relative error is ill-defined where cancellation makes
    y_ref tiny, so the denominator is floored at the rms of the reference."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(y_ref * y_ref))) if y_ref.size else 0.0
    den = np.maximum(np.abs(y_ref), rms)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(y - y_ref) / den)) if y_ref.size else 0.0
