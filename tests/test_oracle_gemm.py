"""Pins for the oracle's masked product Y = (W o M) X.  CPU only."""
import numpy as np
import pytest

import workloads
from oracle import lrbi_oracle as orc
from golden_io import read_sections


def test_worked_example_row_sums():
    g = read_sections("worked_example.txt")
    Y = orc.masked_gemm(g["W"], g["Ia"].astype(np.uint8), np.ones((5, 1)))
    assert np.allclose(Y[:, 0], g["Y1"][:, 0], atol=1e-12)


def test_all_ones_mask_is_plain_matmul():
    rng = np.random.default_rng(0)
    W = rng.standard_normal((37, 53))
    X = rng.standard_normal((53, 9))
    Y = orc.masked_gemm(W, np.ones((37, 53), np.uint8), X)
    assert np.allclose(Y, W @ X, rtol=1e-13, atol=1e-13)


def test_zero_mask_gives_zero():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((5, 6))
    X = rng.standard_normal((6, 2))
    assert not orc.masked_gemm(W, np.zeros((5, 6), np.uint8), X).any()


def test_identity_x_returns_masked_weights():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((8, 12))
    M = (rng.random((8, 12)) < 0.3).astype(np.uint8)
    Y = orc.masked_gemm(W, M, np.eye(12))
    assert np.array_equal(Y, np.where(M == 1, W, 0.0))


def test_against_numpy_where_matmul():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((41, 67))
    M = (rng.random((41, 67)) < 0.2).astype(np.uint8)
    X = rng.standard_normal((67, 5))
    Y = orc.masked_gemm(W, M, X)
    assert np.allclose(Y, np.where(M == 1, W, 0.0) @ X, rtol=1e-12, atol=1e-13)


def test_select_semantics_nan_inf_under_pruned_bits():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((6, 10))
    M = (rng.random((6, 10)) < 0.5).astype(np.uint8)
    X = rng.standard_normal((10, 3))
    ref = orc.masked_gemm(W, M, X)
    Wbad = W.copy()
    Wbad[M == 0] = np.nan
    Wbad[0, np.where(M[0] == 0)[0][:1]] = np.inf
    Y = orc.masked_gemm(Wbad, M, X)
    assert np.isfinite(Y).all() and np.array_equal(Y, ref)


def test_linearity_in_x():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((9, 14))
    M = (rng.random((9, 14)) < 0.4).astype(np.uint8)
    X1, X2 = rng.standard_normal((14, 4)), rng.standard_normal((14, 4))
    lhs = orc.masked_gemm(W, M, 2.0 * X1 - 3.0 * X2)
    rhs = 2.0 * orc.masked_gemm(W, M, X1) - 3.0 * orc.masked_gemm(W, M, X2)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_threads_do_not_change_result():
    rng = np.random.default_rng(6)
    W = rng.standard_normal((64, 80))
    M = (rng.random((64, 80)) < 0.3).astype(np.uint8)
    X = rng.standard_normal((80, 7))
    assert np.array_equal(orc.masked_gemm(W, M, X, threads=1), orc.masked_gemm(W, M, X, threads=4))


def test_empty_row_is_zero():
    W = np.ones((3, 4))
    M = np.array([[1, 0, 1, 0], [0, 0, 0, 0], [1, 1, 1, 1]], np.uint8)
    Y = orc.masked_gemm(W, M, np.ones((4, 1)))
    assert Y[:, 0].tolist() == [2.0, 0.0, 4.0]


def test_c1_end_to_end_shape_and_density():
    d = workloads.make(workloads.CONFIGS["C1"])
    cfg = d["cfg"]
    M = orc.decode_mask(d["Ip01"], d["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Y = orc.masked_gemm(workloads.to_float64(d["W"], cfg.dtype), M, workloads.to_float64(d["X"], cfg.dtype))
    assert Y.shape == (500, 1)
    ref = np.where(M == 1, d["W"].astype(np.float64), 0.0) @ d["X"].astype(np.float64)
    assert orc.rel_err(Y, ref) < 1e-12


def test_rel_err_metric():
    ref = np.array([1.0, -2.0, 0.0, 1e-9])
    rms = np.sqrt(np.mean(ref ** 2))
    y = ref + np.array([0.01, 0.0, 0.0, 0.0])
    assert abs(orc.rel_err(y, ref) - 0.01 / max(1.0, rms)) < 1e-15
    y = ref + np.array([0.0, 0.0, 0.005, 0.0])
    assert abs(orc.rel_err(y, ref) - 0.005 / rms) < 1e-15


def test_lstm_oracle_matches_handwritten_single_step():
    from oracle import lstm
    rng = np.random.default_rng(8)
    H, B = 6, 2
    W = rng.standard_normal((4 * H, 2 * H)) * 0.5
    M = (rng.random((4 * H, 2 * H)) < 0.5).astype(np.uint8)
    xs = rng.standard_normal((2, H, B))
    out = lstm.lstm_sequence([W], [M], xs)
    Wm = np.where(M == 1, W, 0.0)
    h = np.zeros((H, B)); c = np.zeros((H, B))
    for t in range(2):
        z = Wm @ np.concatenate([xs[t], h])
        i, f, g, o = (z[q * H:(q + 1) * H] for q in range(4))
        s = lambda a: 1 / (1 + np.exp(-a))
        c = s(f) * c + s(i) * np.tanh(g)
        h = s(o) * np.tanh(c)
    assert np.allclose(out["h"][0], h, atol=1e-12) and np.allclose(out["c"][0], c, atol=1e-12)
