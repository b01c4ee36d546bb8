"""Pins of oracle/lstm.py (the builder's LSTM cell; Sec. 4 of the paper names the model and prints no equations).
The expected numbers in tests/golden/lstm_cell.txt are worked out by hand from closed forms (gate activations that are
exact rationals), not by running the oracle; a swap of two gates, of the x / h column halves, of gate blocks against
interleaved rows, a sign, or a masked weight read by mistake changes at least one of them.  CPU only."""
import numpy as np

from golden_io import read_sections
from oracle import lstm


def _case():
    g = read_sections("lstm_cell.txt")
    Ws = [g["W1"], g["W2"]]
    Ms = [g["M1"].astype(np.uint8), g["M2"].astype(np.uint8)]
    xs = g["x"].reshape(2, 2, 1)
    c0 = [g["c0_layer1"].reshape(2, 1), np.zeros((2, 1))]
    return g, Ws, Ms, xs, c0


def test_handwritten_two_layer_two_step_case():
    g, Ws, Ms, xs, c0 = _case()
    out = lstm.lstm_sequence(Ws, Ms, xs, c0=c0, record_states=True)
    for t in range(2):
        for l, name in enumerate(("layer1", "layer2")):
            assert np.allclose(out["cs"][t][l][:, 0], g["c_" + name][t], rtol=0, atol=2e-16 * 8), (t, name, "c")
            assert np.allclose(out["hs"][t][l][:, 0], g["h_" + name][t], rtol=0, atol=2e-16 * 8), (t, name, "h")
    assert np.array_equal(out["h"][1], out["hs"][1][1]) and np.array_equal(out["c"][0], out["cs"][1][0])


def test_all_pruned_mask_halves_the_cell_state():
    # z = 0 for every gate: sigm = 1/2, tanh = 0, so c_t = c_{t-1} / 2 exactly and h_t = tanh(c_t) / 2
    H, B = 3, 2
    W = np.full((4 * H, 2 * H), 123.0)
    M = np.zeros((4 * H, 2 * H), np.uint8)
    c0 = np.array([[0.8, -1.6], [0.0, 3.2], [-0.4, 6.4]])
    xs = np.ones((3, H, B))
    out = lstm.lstm_sequence([W], [M], xs, c0=[c0], record_states=True)
    for t in range(3):
        assert np.array_equal(out["cs"][t][0], c0 / 2 ** (t + 1))
    # tanh(0.1) = 0.099667994624955817 (series x - x^3/3 + 2x^5/15 - 17x^7/315 + 62x^9/2835 at x = 0.1)
    assert abs(out["hs"][2][0][0, 0] - 0.5 * 0.099667994624955817) < 1e-16
    # default start: h_0 = c_0 = 0 stays 0 under an all-pruned mask
    out = lstm.lstm_sequence([W], [M], xs)
    assert not out["h"][0].any() and not out["c"][0].any()


def test_planted_mistakes_are_caught_by_the_golden_case():
    """The pin is sharp: each plausible mistake, planted in a copy of the inputs, moves a printed value."""
    g, Ws, Ms, xs, c0 = _case()
    H = 2

    def differs(Ws2, Ms2):
        out = lstm.lstm_sequence(Ws2, Ms2, xs, c0=c0, record_states=True)
        got = np.array([out["hs"][t][l][:, 0] for t in range(2) for l in range(2)])
        want = np.array([g["h_layer%d" % (l + 1)][t] for t in range(2) for l in range(2)])
        return np.abs(got - want).max() > 1e-3

    for a, b in ((0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)):      # two gate blocks exchanged
        for layer in (0, 1):
            Ws2 = [w.copy() for w in Ws]
            Ms2 = [m.copy() for m in Ms]
            for arr in (Ws2[layer], Ms2[layer]):
                tmp = arr[a * H:(a + 1) * H].copy()
                arr[a * H:(a + 1) * H] = arr[b * H:(b + 1) * H]
                arr[b * H:(b + 1) * H] = tmp
            assert differs(Ws2, Ms2), (a, b, layer)
    # x and h column halves exchanged
    assert differs([np.concatenate([w[:, H:], w[:, :H]], axis=1) for w in Ws],
                   [np.concatenate([m[:, H:], m[:, :H]], axis=1) for m in Ms])
    # rows interleaved per unit (i0 f0 g0 o0 i1 ...) instead of gate blocks
    perm = [0, 2, 4, 6, 1, 3, 5, 7]
    assert differs([w[perm] for w in Ws], [m[perm] for m in Ms])
    # mask ignored
    assert differs(Ws, [np.ones_like(m) for m in Ms])
