"""fp64 masked 3 x 3 convolution (test infrastructure only).

TEST INFRASTRUCTURE ONLY: nothing in the product path may import this module.

The paper's convolution rows (Sec. 4: ResNet32, AlexNet conv layers) prune the 4-D filter bank through a 2-D view
of it and leave that view open (Sec. 3.1: the index matrix may be reshaped).  The view taken here, as in the HIP
path: W2d [m, 9 * cin], column (kh * 3 + kw) * cin + ci; the mask has the same shape.  Stride 1, zero padding 1:

    Y[co, b, oh, ow] = sum over kh, kw, ci of  (M * W2d)[co, (kh * 3 + kw) * cin + ci] * act[b, oh + kh - 1, ow + kw - 1, ci]

with act read as zero outside [0, H) x [0, Wd).  The definition is written out as loops over output pixel, filter
tap and channel (`masked_conv3x3_loops`, for small cases) and, for the sizes of the configurations, with the loop
over taps kept and the sums over channels and pixels handed to numpy (`masked_conv3x3`).  Pins, in
tests/test_oracle_conv.py: a hand-computed one-channel case (tests/golden/conv3x3_case.txt), equality of the two
forms, and equality with the masked product on an explicitly unfolded input.
"""
from __future__ import annotations

import numpy as np


def masked_conv3x3_loops(W2d, M, act):
    """Plain loops; act float64 [batch, H, Wd, cin]; returns Y [m, batch * H * Wd]."""
    W2d = np.asarray(W2d, dtype=np.float64)
    act = np.asarray(act, dtype=np.float64)
    batch, H, Wd, cin = act.shape
    m, n = W2d.shape
    if n != 9 * cin or M.shape != (m, n):
        raise ValueError("shape mismatch")
    Y = np.zeros((m, batch * H * Wd), dtype=np.float64)
    for co in range(m):
        for b in range(batch):
            for oh in range(H):
                for ow in range(Wd):
                    s = 0.0
                    for kh in range(3):
                        for kw in range(3):
                            ih, iw = oh + kh - 1, ow + kw - 1
                            if ih < 0 or ih >= H or iw < 0 or iw >= Wd:
                                continue  # zero padding
                            for ci in range(cin):
                                j = (kh * 3 + kw) * cin + ci
                                if M[co, j]:  # a pruned weight is skipped, whatever is stored under it
                                    s += W2d[co, j] * act[b, ih, iw, ci]
                    Y[co, (b * H + oh) * Wd + ow] = s
    return Y


def masked_conv3x3(W2d, M, act):
    """The same sum with numpy doing the channel and pixel sums of each filter tap."""
    W2d = np.asarray(W2d, dtype=np.float64)
    act = np.asarray(act, dtype=np.float64)
    batch, H, Wd, cin = act.shape
    m, n = W2d.shape
    if n != 9 * cin or M.shape != (m, n):
        raise ValueError("shape mismatch")
    Wm = np.where(np.asarray(M) == 1, W2d, 0.0)
    Y = np.zeros((m, batch, H, Wd), dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            # output pixels whose tap (kh, kw) falls inside the image, and the input pixels under it
            oh0, oh1 = max(0, 1 - kh), min(H, H + 1 - kh)
            ow0, ow1 = max(0, 1 - kw), min(Wd, Wd + 1 - kw)
            if oh0 >= oh1 or ow0 >= ow1:
                continue
            window = act[:, oh0 + kh - 1:oh1 + kh - 1, ow0 + kw - 1:ow1 + kw - 1, :]  # [batch, h, w, cin]
            tap = Wm[:, (kh * 3 + kw) * cin:(kh * 3 + kw + 1) * cin]                  # [m, cin]
            Y[:, :, oh0:oh1, ow0:ow1] += np.einsum("oc,bhwc->obhw", tap, window)
    return Y.reshape(m, batch * H * Wd)
