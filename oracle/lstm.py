"""fp64 LSTM recurrence around the masked product (test infrastructure only).

TEST INFRASTRUCTURE ONLY.  The paper names an LSTM as one of its models
(Sec. 4) but prints no cell equations, so this is the builder's own
definition (the usual cell): PARITY UNPINNED by the paper.  The definition
itself is pinned to a handwritten two-layer, two-step case whose gate
activations are exact rationals (tests/golden/lstm_cell.txt, checked in
tests/test_oracle_lstm.py).  It exists to give the 2 x 35 sequential masked
products of the LSTM configuration realistic inputs and to check a
free-running GPU sequence.

Gate matrix rows are [i; f; g; o] blocks of `hidden` rows; columns are
[x_t | h_{t-1}].  z = (W o M) [x_t; h_{t-1}], no bias;
c_t = sigm(z_f) c_{t-1} + sigm(z_i) tanh(z_g);  h_t = sigm(z_o) tanh(c_t);
layer l+1 takes layer l's h_t as x_t;  h_0 = c_0 = 0.
"""
from __future__ import annotations

import numpy as np

from . import lrbi_oracle


def _sigm(z):
    return 1.0 / (1.0 + np.exp(-z))


def lstm_sequence(Ws, Ms, xs, round_input=None, threads: int = 1, h0=None, c0=None, record_states=False):
    """Ws[l] float64 [4H, 2H], Ms[l] uint8 mask, xs float64 [steps, H, B].
    h0, c0: optional per-layer starting states [H, B] (default zero, the configuration's h_0 = c_0 = 0).
    record_states: also return `hs`, `cs`: [steps][layers] copies of h_t, c_t.

    `round_input`, if given, maps the float64 [x; h] block to the values the
    storage dtype can hold (the GPU's product sees its inputs in that dtype);
    the recurrence itself stays in float64.
    Returns dict with per-step per-layer inputs `xh`, pre-activations `z`,
    and final `h`, `c` per layer."""
    layers = len(Ws)
    steps, H, B = xs.shape
    h = [np.zeros((H, B)) if h0 is None else np.array(h0[l], dtype=np.float64) for l in range(layers)]
    c = [np.zeros((H, B)) if c0 is None else np.array(c0[l], dtype=np.float64) for l in range(layers)]
    rec_h = [[None] * layers for _ in range(steps)]
    rec_c = [[None] * layers for _ in range(steps)]
    rec_xh = [[None] * layers for _ in range(steps)]
    rec_z = [[None] * layers for _ in range(steps)]
    for t in range(steps):
        x = xs[t]
        for l in range(layers):
            xh = np.concatenate([x, h[l]], axis=0)
            if round_input is not None:
                xh = round_input(xh)
            z = lrbi_oracle.masked_gemm(Ws[l], Ms[l], xh, threads=threads)
            zi, zf, zg, zo = z[0:H], z[H:2 * H], z[2 * H:3 * H], z[3 * H:4 * H]
            c[l] = _sigm(zf) * c[l] + _sigm(zi) * np.tanh(zg)
            h[l] = _sigm(zo) * np.tanh(c[l])
            rec_xh[t][l] = xh
            rec_z[t][l] = z
            rec_h[t][l], rec_c[t][l] = h[l].copy(), c[l].copy()
            x = h[l]
    out = {"xh": rec_xh, "z": rec_z, "h": h, "c": c}
    if record_states:
        out["hs"], out["cs"] = rec_h, rec_c
    return out
