"""Pins for the oracle's mask decode (Eq. 3 per tile).  CPU only."""
import itertools

import numpy as np
import pytest

import workloads
from oracle import lrbi_oracle as orc
from golden_io import read_sections


def _rand_factors(rng, T, r, c, k, p):
    return ((rng.random((T, r, k)) < p).astype(np.uint8),
            (rng.random((T, k, c)) < p).astype(np.uint8))


def test_worked_example_eq5_to_eq6():
    g = read_sections("worked_example.txt")
    Ip = g["Ip"].astype(np.uint8)[None]
    Iz = g["Iz"].astype(np.uint8)[None]
    Ia = orc.decode_mask(Ip, Iz, 5, 5, 5, 5, 2)
    assert np.array_equal(Ia, g["Ia"].astype(np.uint8))
    # the text: 2 mismatched elements against Eq. 2, both extra keeps
    I = g["I"].astype(np.uint8)
    assert int((Ia != I).sum()) == 2
    assert int(((I == 1) & (Ia == 0)).sum()) == 0


def test_worked_example_thresholds_reproduce_fixture():
    # fixture self-consistency: Eq. 1 -> Eq. 2 at 0.7 and Eq. 4 -> Eq. 5 at (0.5, 0.6), ">="
    g = read_sections("worked_example.txt")
    assert np.array_equal((np.abs(g["W"]) >= 0.7).astype(int), g["I"].astype(int))
    assert np.array_equal((g["Mp"] >= 0.5).astype(int), g["Ip"].astype(int))
    assert np.array_equal((g["Mz"] >= 0.6).astype(int), g["Iz"].astype(int))


def test_or_not_xor_not_sum():
    # overlapping terms: two rank-one terms hit the same entry -> still 1
    Ip = np.array([[[1, 1]]], dtype=np.uint8)
    Iz = np.array([[[1], [1]]], dtype=np.uint8)
    assert orc.decode_mask(Ip, Iz, 1, 1, 1, 1, 2)[0, 0] == 1


@pytest.mark.parametrize("r,c,k", [(1, 1, 1), (2, 2, 1), (2, 3, 2), (3, 2, 2), (3, 3, 1), (2, 2, 2), (3, 3, 2)])
def test_brute_force_set_definition(r, c, k):
    # every factor pair: row i of the mask is the union of the supports of the
    # Iz rows selected by row i of Ip
    nb = r * k + k * c
    for bits in range(1 << nb):
        v = [(bits >> b) & 1 for b in range(nb)]
        Ip = np.array(v[:r * k], dtype=np.uint8).reshape(1, r, k)
        Iz = np.array(v[r * k:], dtype=np.uint8).reshape(1, k, c)
        M = orc.decode_mask(Ip, Iz, r, c, r, c, k)
        for i in range(r):
            support = set()
            for l in range(k):
                if Ip[0, i, l]:
                    support |= {j for j in range(c) if Iz[0, l, j]}
            assert {j for j in range(c) if M[i, j]} == support


@pytest.mark.parametrize("name", ["C1", "C2", "C3a", "C4", "C5"])
def test_integer_product_formulation_on_config_tiles(name):
    # (Ip . Iz over the integers) > 0, tile by tile, with numpy's matmul
    cfg = workloads.CONFIGS[name]
    rng = np.random.default_rng(7)
    gr, gc = 2, 3
    m, n = gr * cfg.r, gc * cfg.c
    Ip, Iz = _rand_factors(rng, gr * gc, cfg.r, cfg.c, cfg.k, cfg.p)
    M = orc.decode_mask(Ip, Iz, m, n, cfg.r, cfg.c, cfg.k)
    for ti in range(gr):
        for tj in range(gc):
            t = ti * gc + tj
            ref = (Ip[t].astype(np.int64) @ Iz[t].astype(np.int64)) > 0
            blk = M[ti * cfg.r:(ti + 1) * cfg.r, tj * cfg.c:(tj + 1) * cfg.c]
            assert np.array_equal(blk.astype(bool), ref)


def test_special_cases():
    rng = np.random.default_rng(3)
    r, c = 7, 11
    # k = 1: outer product (a rectangle)
    u = (rng.random(r) < 0.5).astype(np.uint8)
    v = (rng.random(c) < 0.5).astype(np.uint8)
    M = orc.decode_mask(u.reshape(1, r, 1), v.reshape(1, 1, c), r, c, r, c, 1)
    assert np.array_equal(M, np.outer(u, v))
    # Ip = identity (k = r): mask = Iz
    Iz = (rng.random((1, r, c)) < 0.4).astype(np.uint8)
    M = orc.decode_mask(np.eye(r, dtype=np.uint8)[None], Iz, r, c, r, c, r)
    assert np.array_equal(M, Iz[0])
    # all-ones factors -> all ones; a zero factor -> zero mask
    k = 3
    one_p, one_z = np.ones((1, r, k), np.uint8), np.ones((1, k, c), np.uint8)
    assert orc.decode_mask(one_p, one_z, r, c, r, c, k).all()
    assert not orc.decode_mask(one_p * 0, one_z, r, c, r, c, k).any()
    assert not orc.decode_mask(one_p, one_z * 0, r, c, r, c, k).any()


def test_invariants():
    rng = np.random.default_rng(11)
    r, c, k = 9, 13, 5
    Ip, Iz = _rand_factors(rng, 1, r, c, k, 0.3)
    M = orc.decode_mask(Ip, Iz, r, c, r, c, k)
    # transpose rule: (Ip (x) Iz)^T = Iz^T (x) Ip^T
    Mt = orc.decode_mask(np.ascontiguousarray(Iz.transpose(0, 2, 1)),
                         np.ascontiguousarray(Ip.transpose(0, 2, 1)), c, r, c, r, k)
    assert np.array_equal(Mt, M.T)
    # permuting the rank index in both factors changes nothing
    perm = rng.permutation(k)
    assert np.array_equal(orc.decode_mask(Ip[:, :, perm], Iz[:, perm, :], r, c, r, c, k), M)
    # monotone: setting a factor bit never clears a mask bit
    Ip2 = Ip.copy()
    Ip2[0, 2, 1] = 1
    assert (orc.decode_mask(Ip2, Iz, r, c, r, c, k) >= M).all()
    # at most min(r, 2^k) distinct rows
    assert len({row.tobytes() for row in M}) <= min(r, 2 ** k)
    # nonzero values other than 1 count as set bits
    assert np.array_equal(orc.decode_mask(Ip * 7, Iz * 255, r, c, r, c, k), M)


def test_tiles_are_independent_and_row_major():
    rng = np.random.default_rng(5)
    r, c, k, gr, gc = 4, 6, 3, 3, 2
    m, n = gr * r, gc * c
    Ip, Iz = _rand_factors(rng, gr * gc, r, c, k, 0.4)
    M = orc.decode_mask(Ip, Iz, m, n, r, c, k)
    # flipping tile t's factors to all ones only changes tile t, at the row-major position
    for t in range(gr * gc):
        Ip2, Iz2 = Ip.copy(), Iz.copy()
        Ip2[t] = 1
        Iz2[t] = 1
        M2 = orc.decode_mask(Ip2, Iz2, m, n, r, c, k)
        ti, tj = divmod(t, gc)
        exp = M.copy()
        exp[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c] = 1
        assert np.array_equal(M2, exp)


@pytest.mark.parametrize("name", ["C1", "C2", "C3a", "C4", "C5"])
def test_density_law_eq7(name):
    # Eq. 7 with factor density p in both factors: E[density] = 1 - (1 - p^2)^k.
    # Entries inside a tile are correlated, so the tolerance is empirical, not binomial.
    cfg = workloads.CONFIGS[name]
    rng = np.random.default_rng(2024)
    target_bits = 6_000_000
    T = max(8, target_bits // (cfg.r * cfg.c))
    Ip, Iz = _rand_factors(rng, T, cfg.r, cfg.c, cfg.k, cfg.p)
    M = orc.decode_mask(Ip, Iz, cfg.r, T * cfg.c, cfg.r, cfg.c, cfg.k)
    expect = 1.0 - (1.0 - cfg.p ** 2) ** cfg.k
    got = orc.density(M)
    assert abs(got - expect) < 0.004, (got, expect)
    # the GF(2) (xor) product would give (1 - (1 - 2 p^2)^k) / 2: must be told apart for k*p^2 large enough
    xor_density = (1.0 - (1.0 - 2 * cfg.p ** 2) ** cfg.k) / 2.0
    if abs(xor_density - expect) > 0.008:
        assert abs(got - xor_density) > 0.004


def test_workload_values_from_baseline_table():
    exp = {"C1": 0.0985, "C2": 0.0976, "C3a": 0.1090, "C4": 0.1096, "C5": 0.2786}
    for name, d in exp.items():
        cfg = workloads.CONFIGS[name]
        assert abs((1 - (1 - cfg.p ** 2) ** cfg.k) - d) < 5e-4


def test_rejects_bad_shapes():
    Ip = np.zeros((1, 2, 1), np.uint8)
    Iz = np.zeros((1, 1, 2), np.uint8)
    with pytest.raises(ValueError):
        orc.decode_mask(Ip, Iz, 3, 2, 2, 2, 1)
    with pytest.raises(ValueError):
        orc.decode_mask(Ip, Iz, 2, 2, 2, 2, 2)
