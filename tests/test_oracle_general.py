"""Pins of the oracle for tiles that do not divide the matrix and for per-tile ranks (Sec. 3.1:
every submatrix is factorised on its own and may choose its own rank).  Each check reduces the general case
to something fixed elsewhere: the set definition written out in plain Python, or the uniform, dividing case
that the printed example and the brute-force tests already pin."""
import numpy as np
import pytest

from oracle import lrbi_oracle as orc


def _factors(rng, T, r, c, k, p=0.3):
    return (rng.random((T, r, k)) < p).astype(np.uint8), (rng.random((T, k, c)) < p).astype(np.uint8)


def _brute(Ip, Iz, m, n, r, c, k, rank=None):
    tile_cols = -(-n // c)
    M = np.zeros((m, n), np.uint8)
    for i in range(m):
        for j in range(n):
            t = (i // r) * tile_cols + j // c
            kt = k if rank is None else int(rank[t])
            M[i, j] = int(any(Ip[t, i % r, l] and Iz[t, l, j % c] for l in range(kt)))
    return M


@pytest.mark.parametrize("m,n,r,c,k", [(7, 9, 3, 4, 2), (10, 10, 4, 4, 3), (5, 13, 5, 5, 4), (11, 6, 4, 6, 2)])
def test_edge_tiles_against_the_set_definition(m, n, r, c, k):
    rng = np.random.default_rng(m * 100 + n)
    T = orc.num_tiles(m, n, r, c)
    Ip, Iz = _factors(rng, T, r, c, k)
    assert np.array_equal(orc.decode_mask(Ip, Iz, m, n, r, c, k), _brute(Ip, Iz, m, n, r, c, k))


@pytest.mark.parametrize("m,n,r,c,k", [(70, 90, 32, 40, 5), (100, 129, 64, 64, 9), (33, 64, 32, 64, 3)])
def test_edge_tiles_are_the_crop_of_the_padded_matrix(m, n, r, c, k):
    """Cutting tiles off at the edge = decoding the matrix padded up to whole tiles (a dividing tiling, pinned
    elsewhere) and keeping its top-left m x n corner; what lies in the cut-off part of the factors is irrelevant."""
    rng = np.random.default_rng(7)
    T = orc.num_tiles(m, n, r, c)
    Ip, Iz = _factors(rng, T, r, c, k)
    mp, np_ = -(-m // r) * r, -(-n // c) * c
    full = orc.decode_mask(Ip, Iz, mp, np_, r, c, k)
    assert np.array_equal(orc.decode_mask(Ip, Iz, m, n, r, c, k), full[:m, :n])


def test_per_tile_rank_against_the_set_definition_and_tile_by_tile():
    rng = np.random.default_rng(11)
    m, n, r, c, k = 12, 15, 4, 5, 6
    T = orc.num_tiles(m, n, r, c)
    Ip, Iz = _factors(rng, T, r, c, k, p=0.35)
    rank = rng.integers(0, k + 1, size=T).astype(np.int32)
    rank[0], rank[1] = 0, k      # both extremes occur
    M = orc.decode_mask(Ip, Iz, m, n, r, c, k, tile_rank=rank)
    assert np.array_equal(M, _brute(Ip, Iz, m, n, r, c, k, rank))
    # tile by tile: a single-tile matrix with the truncated factors at the tile's own (uniform) rank
    tile_cols = n // c
    for t in range(T):
        ti, tj = divmod(t, tile_cols)
        kt = int(rank[t])
        block = M[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c]
        if kt == 0:
            assert not block.any()
        else:
            one = orc.decode_mask(Ip[t:t + 1, :, :kt], Iz[t:t + 1, :kt, :], r, c, r, c, kt)
            assert np.array_equal(block, one)
    # and it is the uniform decode of factors whose unused ranks are cleared
    Ip0, Iz0 = Ip.copy(), Iz.copy()
    for t in range(T):
        Ip0[t, :, rank[t]:] = 0
        Iz0[t, rank[t]:, :] = 0
    assert np.array_equal(M, orc.decode_mask(Ip0, Iz0, m, n, r, c, k))


def test_index_size_closed_forms():
    # dividing, uniform: tiles k (r + c), the form used for Tables 1 and 3
    assert orc.index_bits(4096, 9216, 256, 256, 16) == 16 * 36 * 16 * 512
    # edge tiles: every tile column stores m rows of I_p, every tile row n columns of I_z
    for (m, n, r, c, k) in [(70, 90, 32, 40, 5), (500, 800, 128, 96, 4), (1, 1, 8, 8, 3)]:
        assert orc.index_bits(m, n, r, c, k) == k * (-(-n // c) * m + -(-m // r) * n)
    # per-tile rank: linear in each tile's rank
    rank = np.array([1, 2, 3, 4, 5, 6], np.int32)
    assert orc.index_bits(8, 12, 4, 4, 6, tile_rank=rank) == int(rank.sum()) * 8
    # the ResNet-32 setting of Sec. 3: ranks chosen per layer group on 576 x 512-like tiles stay additive
    a = orc.index_bits(576, 1024, 576, 512, 256, tile_rank=np.array([145, 256], np.int32))
    assert a == (145 + 256) * (576 + 512)


def test_candidate_cost_on_edge_tiles():
    rng = np.random.default_rng(3)
    m, n, r, c = 7, 10, 3, 4
    W = rng.normal(size=(m, n))
    M = (rng.random((m, n)) < 0.4).astype(np.uint8)
    kept, cost = orc.candidate_cost(W, 0.5, M, r, c)
    tile_cols = -(-n // c)
    for t in range(orc.num_tiles(m, n, r, c)):
        ti, tj = divmod(t, tile_cols)
        Wt, Mt = W[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c], M[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c]
        assert kept[t] == Mt.sum()
        assert abs(cost[t] - np.abs(Wt)[(np.abs(Wt) >= 0.5) & (Mt == 0)].sum()) < 1e-12
    assert kept.sum() == M.sum()
