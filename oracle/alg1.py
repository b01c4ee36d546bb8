"""CPU oracle for the threshold search of Algorithm 1 (arXiv 1905.05686, Sec. 2.1), tile by tile.

TEST INFRASTRUCTURE ONLY: plain loops over tiles, S_p values and bisection steps, in the order
of the printed algorithm; every candidate is evaluated with the plain C oracle (threshold,
decode, ones, cost).  Shares no code with the GPU library.

Given W, the real-valued non-negative factors (M_p, M_z) of every tile (from any NMF; given
here), the rank k and the target sparsity S, the algorithm sweeps the sparsity S_p of I_p; for
each S_p it starts S_z at the value Eq. 7 predicts, S_z = (S^(1/k) - S_p) / (1 - S_p), and
adjusts it by binary search until the sparsity S_a of I_a = I_p (x) I_z is as close to S as it
gets; the candidate's cost is the summed magnitude of the weights that magnitude pruning
keeps and I_a prunes; the cheapest candidate wins.

Readings where the paper is silent (the same ones as the library's header states):
  * "convert with (S_p, S_z)": the threshold is the entry of the tile's sorted factor at index
    round(S * count): entries below it become 0, so about a fraction S of them.  Index = count
    (everything pruned) gives threshold +inf.
  * the step of the sweep is the caller's list of S_p values, visited in the given order.
  * "adjust S_z": bisection on [0, 1]: first probe at the Eq. 7 value (clipped to [0, 1]); if I_a
    has more ones than the target the lower end moves up to the probe, otherwise the upper end
    moves down; next probe = midpoint; a fixed number of probes; the probe whose number of ones
    is closest to the target represents this S_p (first one on ties).
  * "S_a ~ S": |ones - target ones| <= tolerance makes a candidate eligible.  An eligible
    candidate beats an ineligible one; two eligible ones compare by cost (first wins ties); two
    ineligible ones by distance to the target (first wins ties).
  * target ones = round((1 - S) r c); all sparsity comparisons are made on these integers.
  * the cost is summed over the magnitudes the factorisation saw (Sec. 3.2 manipulates the magnitudes "to keep
    the definition of Cost"): `method`, `amplify` as in oracle/nmf.py (1 none, 2 squared, 3 amplified kept set).
  * a tile cut off at the matrix edge is searched as the smaller tile it is: its target, its quantiles and
    its cost use only the part inside the matrix.
Pins: tests/test_oracle_search.py (the printed example is recovered: S_p = 0.5 finds Eq. 5 and
Eq. 6 with cost 0; planted two-level factors are recovered exactly; the result is always one of
the visited candidates and re-evaluates to the reported numbers).
"""
import math

import numpy as np

from . import lrbi_oracle as orc


def quantile_index(sparsity: float, count: int) -> int:
    i = int(math.floor(sparsity * count + 0.5))
    return min(max(i, 0), count)


def threshold_at(sorted_values: np.ndarray, index: int) -> np.float32:
    return np.float32(np.inf) if index >= sorted_values.size else np.float32(sorted_values[index])


def initial_sz(S: float, k: int, sp: float) -> float:
    """Eq. 7 solved for S_z, clipped to [0, 1]."""
    if sp >= 1.0:
        return 0.0
    v = (S ** (1.0 / k) - sp) / (1.0 - sp)
    return min(max(v, 0.0), 1.0)


def search_thresholds(W, w_threshold, Mp, Mz, r, c, S, sp_values, steps, tolerance, method=1, amplify=1.0):
    """Returns per tile: Tp, Tz (float32), kept (uint64), cost (float64) of the winning candidate."""
    W = np.asarray(W, dtype=np.float64)
    Mp = np.asarray(Mp, dtype=np.float32)
    Mz = np.asarray(Mz, dtype=np.float32)
    m, n = W.shape
    T, _, k = Mp.shape
    tile_cols = -(-n // c)
    if T != -(-m // r) * tile_cols:
        raise ValueError("one pair of factors per tile")
    out_tp = np.zeros(T, np.float32)
    out_tz = np.zeros(T, np.float32)
    out_kept = np.zeros(T, np.uint64)
    out_cost = np.zeros(T, np.float64)
    for t in range(T):
        ti, tj = divmod(t, tile_cols)
        # the tile's part inside the matrix (an edge tile is cut off): rt x ct; only the factor entries that
        # belong to it take part, in the quantiles as well
        Wt = W[ti * r:(ti + 1) * r, tj * c:(tj + 1) * c]
        rt, ct = Wt.shape
        Mp_t = np.ascontiguousarray(Mp[t, :rt, :])[None]
        Mz_t = np.ascontiguousarray(Mz[t, :, :ct])[None]
        target = int(math.floor((1.0 - S) * rt * ct + 0.5))
        sp_sorted = np.sort(Mp_t.reshape(-1))
        sz_sorted = np.sort(Mz_t.reshape(-1))
        best = None  # (eligible, cost, diff, Tp, Tz, kept)
        for sp in sp_values:
            tp = threshold_at(sp_sorted, quantile_index(sp, sp_sorted.size))
            lo, hi = 0.0, 1.0
            sz = initial_sz(S, k, sp)
            rep = None  # (diff, Tz, kept, cost): the probe closest to the target
            for _ in range(steps):
                tz = threshold_at(sz_sorted, quantile_index(sz, sz_sorted.size))
                Ip, Iz = orc.threshold_factors(Mp_t, Mz_t, np.array([tp], np.float32), np.array([tz], np.float32))
                Ia = orc.decode_mask(Ip, Iz, rt, ct, rt, ct, k)
                kept, cost = orc.candidate_cost(Wt, w_threshold, Ia, rt, ct, method, amplify)
                kept, cost = int(kept[0]), float(cost[0])
                diff = abs(kept - target)
                if rep is None or diff < rep[0]:
                    rep = (diff, tz, kept, cost)
                if kept > target:
                    lo = sz
                else:
                    hi = sz
                sz = 0.5 * (lo + hi)
            diff, tz, kept, cost = rep
            eligible = diff <= tolerance
            if best is None:
                better = True
            elif eligible != best[0]:
                better = eligible
            elif eligible:
                better = cost < best[1]
            else:
                better = diff < best[2]
            if better:
                best = (eligible, cost, diff, tp, tz, kept)
        out_tp[t], out_tz[t], out_kept[t], out_cost[t] = best[3], best[4], best[5], best[1]
    return out_tp, out_tz, out_kept, out_cost
