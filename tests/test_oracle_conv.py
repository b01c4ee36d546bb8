"""The masked 3 x 3 convolution oracle (oracle/conv.py) against a hand-computed case, against its own loop form,
and against the masked product on an explicitly unfolded input."""
import numpy as np

from golden_io import read_sections
from oracle import conv as conv_oracle
from oracle import lrbi_oracle as orc


def _unfold(act):
    """X [9 * cin, batch * H * Wd] written independently of the oracle: pad, then copy the nine shifted images."""
    batch, H, Wd, cin = act.shape
    p = np.pad(act, ((0, 0), (1, 1), (1, 1), (0, 0)))
    X = np.empty((9 * cin, batch * H * Wd))
    for kh in range(3):
        for kw in range(3):
            shifted = p[:, kh:kh + H, kw:kw + Wd, :]                       # [batch, H, Wd, cin]
            X[(kh * 3 + kw) * cin:(kh * 3 + kw + 1) * cin] = shifted.reshape(-1, cin).T
    return X


def test_hand_computed_case():
    g = read_sections("conv3x3_case.txt")
    act = g["act"].reshape(1, 3, 3, 1)
    M = g["M"].astype(np.uint8)
    for f in (conv_oracle.masked_conv3x3_loops, conv_oracle.masked_conv3x3):
        assert np.array_equal(f(g["W"], M, act), g["Y"]), f.__name__
    # planted mistakes on the oracle's side: each must change the result
    assert not np.array_equal(conv_oracle.masked_conv3x3(g["W"], M, act.transpose(0, 2, 1, 3)), g["Y"])
    flipped = g["W"].reshape(2, 3, 3)[:, ::-1, ::-1].reshape(2, 9)
    assert not np.array_equal(conv_oracle.masked_conv3x3(flipped, M.reshape(2, 3, 3)[:, ::-1, ::-1].reshape(2, 9), act),
                              g["Y"])
    assert not np.array_equal(conv_oracle.masked_conv3x3(g["W"], np.ones_like(M), act), g["Y"])


def test_loop_form_and_tap_form_agree():
    rng = np.random.default_rng(0)
    for (batch, H, Wd, cin, m) in [(2, 4, 5, 3, 6), (1, 1, 1, 2, 3), (3, 2, 7, 1, 4)]:
        act = rng.standard_normal((batch, H, Wd, cin))
        W = rng.standard_normal((m, 9 * cin))
        M = (rng.random((m, 9 * cin)) < 0.4).astype(np.uint8)
        a, b = conv_oracle.masked_conv3x3_loops(W, M, act), conv_oracle.masked_conv3x3(W, M, act)
        assert np.allclose(a, b, rtol=0, atol=1e-12)


def test_equals_the_masked_product_on_the_unfolded_input():
    rng = np.random.default_rng(1)
    batch, H, Wd, cin, m = 3, 6, 5, 8, 10
    act = rng.standard_normal((batch, H, Wd, cin))
    W = rng.standard_normal((m, 9 * cin))
    M = (rng.random((m, 9 * cin)) < 0.3).astype(np.uint8)
    Y = conv_oracle.masked_conv3x3(W, M, act)
    ref = orc.masked_gemm(W, M, _unfold(act))
    assert np.allclose(Y, ref, rtol=0, atol=1e-12)
    # NaN under a pruned bit stays out (select, not multiply)
    Wp = np.where(M == 1, W, np.nan)
    assert np.array_equal(conv_oracle.masked_conv3x3(Wp, M, act), Y)
