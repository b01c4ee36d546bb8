"""Pins for the oracle's threshold search of Algorithm 1 (Sec. 2.1).  CPU only."""
import numpy as np
import pytest

from oracle import alg1
from oracle import lrbi_oracle as orc
from golden_io import read_sections


def test_index_and_initial_sz():
    # Eq. 7 and its inverse: S = (1 - (1 - S_p)(1 - S_z))^k  <->  S_z = (S^(1/k) - S_p) / (1 - S_p)
    for S, k, sp in ((0.9, 16, 0.3), (0.48, 2, 0.5), (0.95, 4, 0.1)):
        sz = alg1.initial_sz(S, k, sp)
        assert (1.0 - (1.0 - sp) * (1.0 - sz)) ** k == pytest.approx(S, rel=1e-12)
    assert alg1.initial_sz(0.5, 2, 0.9) == 0.0            # S_p alone already exceeds S^(1/k): clipped
    assert alg1.quantile_index(0.5, 10) == 5 and alg1.quantile_index(1.0, 10) == 10 and alg1.quantile_index(0.0, 10) == 0
    assert alg1.threshold_at(np.float32([1, 2, 3]), 3) == np.inf


def test_worked_example_is_recovered():
    # Sec. 2.1: with S_p = 0.5 the thresholds behind Eq. 5 give S_a = 0.40 (15 ones, Eq. 6) and lose none of
    # the weights of Eq. 2.  Searching for S = 0.40 from Eq. 4 must find exactly these factors.
    g = read_sections("worked_example.txt")
    Mp = g["Mp"].astype(np.float32)[None]
    Mz = g["Mz"].astype(np.float32)[None]
    Tp, Tz, kept, cost = alg1.search_thresholds(g["W"], 0.7, Mp, Mz, 5, 5, 0.40, [0.5], steps=6, tolerance=0)
    Ip, Iz = orc.threshold_factors(Mp, Mz, Tp, Tz)
    assert np.array_equal(Ip[0], g["Ip"].astype(np.uint8)) and np.array_equal(Iz[0], g["Iz"].astype(np.uint8))
    assert int(kept[0]) == 15 and cost[0] == 0.0
    # sweeping other S_p values as well cannot do better than cost 0 at the target sparsity
    Tp2, Tz2, kept2, cost2 = alg1.search_thresholds(g["W"], 0.7, Mp, Mz, 5, 5, 0.40, [0.0, 0.2, 0.5, 0.7], steps=6,
                                                    tolerance=0)
    assert int(kept2[0]) == 15 and cost2[0] == 0.0


def test_planted_two_level_factors_are_recovered():
    # factors whose entries take two values only: every threshold between them yields the planted bits, so a sweep
    # that contains a S_p at or above the planted sparsity of I_p must return the planted mask with cost 0
    rng = np.random.default_rng(4)
    r, c, k = 12, 16, 3
    Ip = (rng.random((1, r, k)) < 0.4).astype(np.uint8)
    Iz = (rng.random((1, k, c)) < 0.4).astype(np.uint8)
    Mp = np.where(Ip == 1, 0.9, 0.1).astype(np.float32)
    Mz = np.where(Iz == 1, 0.8, 0.2).astype(np.float32)
    Ia = orc.decode_mask(Ip, Iz, r, c, r, c, k)
    W = np.where(Ia == 1, 2.0, 0.01) * rng.choice([-1.0, 1.0], (r, c))
    S = 1.0 - Ia.mean()
    sp_planted = 1.0 - Ip.mean()
    Tp, Tz, kept, cost = alg1.search_thresholds(W, 1.0, Mp, Mz, r, c, S, [0.0, sp_planted, 0.95], steps=10, tolerance=0)
    assert int(kept[0]) == int(Ia.sum()) and cost[0] == 0.0
    Ip2, Iz2 = orc.threshold_factors(Mp, Mz, Tp, Tz)
    assert np.array_equal(orc.decode_mask(Ip2, Iz2, r, c, r, c, k), Ia)


def test_result_is_a_visited_candidate_and_reevaluates():
    rng = np.random.default_rng(9)
    m, n, r, c, k = 32, 48, 16, 24, 4
    T = 4
    W = rng.normal(0, 1, (m, n))
    Mp = rng.random((T, r, k), dtype=np.float32)
    Mz = rng.random((T, k, c), dtype=np.float32)
    S, tol = 0.8, 8
    sp_values = [0.0, 0.25, 0.5, 0.75]
    Tp, Tz, kept, cost = alg1.search_thresholds(W, 1.0, Mp, Mz, r, c, S, sp_values, steps=8, tolerance=tol)
    # thresholds are entries of the tile's factors (or +inf), Tp belongs to one of the swept S_p values
    for t in range(T):
        sp_sorted = np.sort(Mp[t].reshape(-1))
        assert any(Tp[t] == alg1.threshold_at(sp_sorted, alg1.quantile_index(sp, sp_sorted.size)) for sp in sp_values)
        assert np.isinf(Tz[t]) or Tz[t] in Mz[t]
    # re-evaluating the returned thresholds gives the returned numbers
    Ip, Iz = orc.threshold_factors(Mp, Mz, Tp, Tz)
    M = orc.decode_mask(Ip, Iz, m, n, r, c, k)
    kept2, cost2 = orc.candidate_cost(W, 1.0, M, r, c)
    assert np.array_equal(kept, kept2) and np.array_equal(cost, cost2)
    # more bisection steps never end farther from the target, tile by tile, when only one S_p is swept
    target = round((1 - S) * r * c)
    _, _, k4, _ = alg1.search_thresholds(W, 1.0, Mp, Mz, r, c, S, [0.25], steps=4, tolerance=0)
    _, _, k12, _ = alg1.search_thresholds(W, 1.0, Mp, Mz, r, c, S, [0.25], steps=12, tolerance=0)
    assert np.all(np.abs(k12.astype(np.int64) - target) <= np.abs(k4.astype(np.int64) - target))


def test_brute_force_over_all_thresholds_on_a_tiny_tile():
    # on a tiny tile every pair of thresholds can be tried: the search result must be one of those candidates, and
    # among the candidates as close to the target as the one it reports, none visited by the search is cheaper
    rng = np.random.default_rng(2)
    r, c, k = 4, 5, 2
    W = rng.normal(0, 1, (r, c))
    Mp = rng.random((1, r, k), dtype=np.float32)
    Mz = rng.random((1, k, c), dtype=np.float32)
    S = 0.6
    target = round((1 - S) * r * c)
    sp_values = [i / 8 for i in range(8)]
    Tp, Tz, kept, cost = alg1.search_thresholds(W, 0.5, Mp, Mz, r, c, S, sp_values, steps=8, tolerance=0)
    cands = {}
    for tp in list(np.sort(Mp.reshape(-1))) + [np.float32(np.inf)]:
        for tz in list(np.sort(Mz.reshape(-1))) + [np.float32(np.inf)]:
            Ip, Iz = orc.threshold_factors(Mp, Mz, np.float32([tp]), np.float32([tz]))
            M = orc.decode_mask(Ip, Iz, r, c, r, c, k)
            kk, cc = orc.candidate_cost(W, 0.5, M, r, c)
            cands[(float(tp), float(tz))] = (int(kk[0]), float(cc[0]))
    assert (float(Tp[0]), float(Tz[0])) in cands
    assert cands[(float(Tp[0]), float(Tz[0]))] == (int(kept[0]), float(cost[0]))
    # For a fixed T_p the number of ones falls monotonically as T_z rises, and 8 halvings of [0, 1] resolve the 11
    # possible T_z of this tile, so the bisection reaches the T_z closest to the target for every swept S_p.  The
    # result must therefore be exactly as close to the target as brute force over (swept T_p) x (every T_z) gets.
    sorted_p = np.sort(Mp.reshape(-1))
    swept_tp = {float(alg1.threshold_at(sorted_p, alg1.quantile_index(sp, sorted_p.size))) for sp in sp_values}
    assert float(Tp[0]) in swept_tp
    reach = {tp: min(abs(v[0] - target) for (tp2, _), v in cands.items() if tp2 == tp) for tp in swept_tp}
    assert abs(int(kept[0]) - target) == min(reach.values())
    if min(reach.values()) == 0:
        # eligible winners compare by cost: no swept T_p whose every target-hitting T_z is cheaper can have lost
        for tp, d in reach.items():
            if d == 0:
                worst = max(v[1] for (tp2, _), v in cands.items() if tp2 == tp and v[0] == target)
                assert float(cost[0]) <= worst


def test_cut_off_tiles_are_searched_as_the_smaller_tiles_they_are():
    """A matrix whose last tile row and column stick out: every tile's result equals the search on that tile alone,
    as a one-tile matrix of its cut-off shape with the matching part of the factors (a case the pins above cover)."""
    rng = np.random.default_rng(21)
    m, n, r, c, k = 11, 14, 4, 5, 3
    T = 3 * 3
    W = rng.normal(size=(m, n))
    Mp = rng.random((T, r, k)).astype(np.float32)
    Mz = rng.random((T, k, c)).astype(np.float32)
    sweep, steps, tol, S = [0.3, 0.6, 0.8], 6, 1, 0.6
    tp, tz, kept, cost = alg1.search_thresholds(W, 0.8, Mp, Mz, r, c, S, sweep, steps, tol)
    for t in range(T):
        ti, tj = divmod(t, 3)
        Wt = W[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c]
        rt, ct = Wt.shape
        one = alg1.search_thresholds(Wt, 0.8, Mp[t:t + 1, :rt, :], Mz[t:t + 1, :, :ct], rt, ct, S, sweep, steps, tol)
        assert (tp[t], tz[t], kept[t]) == (one[0][0], one[1][0], one[2][0]) and cost[t] == one[3][0]
