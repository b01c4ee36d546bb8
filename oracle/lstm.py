"""fp64 LSTM recurrence around the masked product (test infrastructure only).

The paper names an LSTM as one of its models (Sec. 4) but prints no cell
equations, so this is the builder's own definition: PARITY UNPINNED by the
paper.  It exists to give the 2 x 35 sequential masked products of the LSTM
configuration realistic inputs and to check a free-running GPU sequence.

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


def lstm_sequence(Ws, Ms, xs, round_input=None, threads: int = 1):
    """Ws[l] float64 [4H, 2H], Ms[l] uint8 mask, xs float64 [steps, H, B].

    `round_input`, if given, maps the float64 [x; h] block to the values the
    storage dtype can hold (the GPU's product sees its inputs in that dtype);
    the recurrence itself stays in float64.
    Returns dict with per-step per-layer inputs `xh`, pre-activations `z`,
    and final `h`, `c` per layer."""
    layers = len(Ws)
    steps, H, B = xs.shape
    h = [np.zeros((H, B)) for _ in range(layers)]
    c = [np.zeros((H, B)) for _ in range(layers)]
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
            x = h[l]
    return {"xh": rec_xh, "z": rec_z, "h": h, "c": c}
