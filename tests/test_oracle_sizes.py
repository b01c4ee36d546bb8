"""Pins for the index-size accounting (Sec. 2.2, Tables 1 and 3).  CPU only."""
import numpy as np
import pytest

import workloads
from oracle import lrbi_oracle as orc
from golden_io import read_rows


def test_printed_sizes_and_ratios():
    for kind, m, n, r, c, k, val, unit in read_rows("index_sizes.txt"):
        m, n, r, c, k, val = int(m), int(n), int(r), int(c), int(k), float(val)
        if kind == "ratio":
            got = orc.compression_ratio(m, n, r, c, k)
            assert abs(got - val) <= 0.05 + 1e-9, (m, n, k, got, val)
        else:
            bits = orc.dense_bits(m, n) if kind == "dense" else orc.index_bits(m, n, r, c, k)
            per = 8 * 1000 if unit == "kB" else 8 * 1024
            tol = 0.05 if unit == "kB" else 1e-9
            assert abs(bits / per - val) <= tol, (kind, m, n, k, bits / per, val)


def test_ratio_matches_formula_mn_over_k_m_plus_n():
    for k in (1, 3, 16, 145, 256):
        assert orc.compression_ratio(800, 500, 800, 500, k) == pytest.approx(800 * 500 / (k * 1300))


def test_tiling_equivalence_fig4():
    # 1x1 tiles with k=128, 2x2 with k=64, 4x4 with k=32 cost the same (Sec. 3.1, FC1 500x800)
    a = orc.index_bits(500, 800, 500, 800, 128)
    b = orc.index_bits(500, 800, 250, 400, 64)
    c = orc.index_bits(500, 800, 125, 200, 32)
    assert a == b == c == 128 * 1300


def test_config_values():
    exp = {"C1": (32000, 400000), "C2": (4718592, 37748736), "C3a": (2097152, 16777216),
           "C4": (960000, 18000000), "C5": (73728, 589824)}
    for name, (lr, dn) in exp.items():
        cfg = workloads.CONFIGS[name]
        assert orc.index_bits(cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) == lr
        assert orc.dense_bits(cfg.m, cfg.n) == dn
        assert cfg.tiles * cfg.k * (cfg.r + cfg.c) == lr


def test_index_bits_equals_factor_element_count():
    cfg = workloads.CONFIGS["C1"]
    d = workloads.make(cfg, want_w=False, want_x=False)
    assert d["Ip01"].size + d["Iz01"].size == orc.index_bits(cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)


def test_csr_bits_builder_formula():
    # parity unpinned by the paper; only the builder's stated accounting is checked
    assert orc.csr_bits(20000, 500, 16, 32) == 20000 * 16 + 501 * 32
    M = np.eye(4, dtype=np.uint8)
    assert orc.popcount(M) == 4 and orc.density(M) == 0.25


def test_csr_bits_counts_the_arrays_of_a_library_csr_matrix():
    # the accounting (one column index per kept weight, m + 1 row pointers) against the arrays scipy actually builds
    import scipy.sparse
    rng = np.random.default_rng(3)
    for (m, n, p) in [(7, 5, 0.3), (50, 80, 0.05), (1, 9, 1.0), (12, 12, 0.0)]:
        dense = (rng.random((m, n)) < p).astype(np.float32)
        csr = scipy.sparse.csr_matrix(dense)
        for idx_bits, ptr_bits in [(16, 32), (8, 16)]:
            assert orc.csr_bits(int(csr.nnz), m, idx_bits, ptr_bits) == csr.indices.size * idx_bits + csr.indptr.size * ptr_bits


def test_invalid_shapes():
    with pytest.raises(ValueError):
        orc.index_bits(10, 10, 0, 5, 2)
    with pytest.raises(ValueError):
        orc.index_bits(10, 10, 5, 5, 0)
    # tiles that do not divide the matrix are cut off at its edge (sizes in tests/test_oracle_general.py)
    assert orc.index_bits(10, 10, 3, 5, 2) == 2 * (2 * 10 + 4 * 10)
