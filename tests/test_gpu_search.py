"""GPU parity of lrbi_search_thresholds (threshold search of Algorithm 1, Sec. 2.1) against the oracle's
plain tile-by-tile search."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import alg1
from oracle import lrbi_oracle as orc
from gpu_util import desc_of, dev, to_device

pytestmark = pytest.mark.gpu


def _cfg(m, n, r, c, k, dtype, seed, p=0.2):
    return workloads.Config("t", m, n, r, c, k, p, 1, dtype, 0.05, seed)


def _run(cfg, S, sp_values, steps, tolerance, want_factors=True, method=1, amplify=1.0):
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    W = to_device(data["W"], cfg.dtype)
    t = lambda a: torch.from_numpy(a).to(dev())
    out = lrbi.search_thresholds(desc_of(cfg), W, f["w_threshold"], t(f["Mp"]), t(f["Mz"]), S, sp_values, steps,
                                 tolerance, want_factors=want_factors, method=method, amplify=amplify)
    torch.cuda.synchronize()
    return W64, f, out


def _check(cfg, S, sp_values, steps, tolerance, method=1, amplify=1.0):
    W64, f, (Tp, Tz, kept, cost, ip, iz) = _run(cfg, S, sp_values, steps, tolerance, method=method, amplify=amplify)
    amplify = float(np.float32(amplify))
    ref_tp, ref_tz, ref_kept, ref_cost = alg1.search_thresholds(W64, f["w_threshold"], f["Mp"], f["Mz"], cfg.r, cfg.c, S,
                                                                sp_values, steps, tolerance, method, amplify)
    Tp, Tz = Tp.cpu().numpy(), Tz.cpu().numpy()
    kept, cost = kept.cpu().numpy().astype(np.uint64), cost.cpu().numpy()
    # 1. whatever was chosen re-evaluates, by the oracle, to the numbers reported: counts exact, cost a
    #    double-precision sum of the same terms in another order
    Ip, Iz = orc.threshold_factors(f["Mp"], f["Mz"], Tp, Tz)
    M = orc.decode_mask(Ip, Iz, cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    k2, c2 = orc.candidate_cost(W64, f["w_threshold"], M, cfg.r, cfg.c, method, amplify)
    assert np.array_equal(k2, kept)
    assert np.all(np.abs(c2 - cost) <= 1e-12 * np.maximum(c2, 1.0))
    ip_ref, iz_ref = lrbi.pack_factors(desc_of(cfg), Ip, Iz)
    assert np.array_equal(ip.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(ip_ref).view(np.uint32).reshape(-1))
    assert np.array_equal(iz.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(iz_ref).view(np.uint32).reshape(-1))
    # 2. the choice is the oracle's.  The thresholds are entries of the factors and the counts integers: exact.
    #    Only where two candidates' costs agree to rounding may the other one win; then the costs still agree.
    same = (Tp == ref_tp) & (Tz == ref_tz)
    assert np.all(np.abs(cost - ref_cost) <= 1e-12 * np.maximum(ref_cost, 1.0)), (cost, ref_cost)
    assert np.array_equal(kept[same], ref_kept[same])
    # a tile with another winner: same cost (asserted above) and the same standing against the target (whole tiles
    # here), so the two candidates are a tie that the rounding of the sums decided
    target = int(np.floor((1.0 - S) * cfg.r * cfg.c + 0.5))
    d_gpu = np.abs(kept.astype(np.int64) - target)
    d_ref = np.abs(ref_kept.astype(np.int64) - target)
    if cfg.m % cfg.r == 0 and cfg.n % cfg.c == 0:
        other = ~same
        assert np.array_equal(d_gpu[other] <= tolerance, d_ref[other] <= tolerance)
        inel = other & (d_ref > tolerance)
        assert np.array_equal(d_gpu[inel], d_ref[inel])
    return same


SWEEP = [0.0, 0.3, 0.5, 0.7, 0.9]


@pytest.mark.parametrize("method,amplify", [(2, 1.0), (3, 1.0 / (1.0 - 0.91))])
def test_search_with_manipulated_cost(method, amplify):
    """Sec. 3.2: the search minimises the cost over the manipulated magnitudes, as the oracle does."""
    print("search manipulated", method, amplify, flush=True)
    cfg = _cfg(256, 512, 128, 256, 16, "bf16", 3)
    _check(cfg, 0.91, SWEEP, 9, 64, method=method, amplify=amplify)
    cfg = _cfg(200, 300, 100, 100, 4, "f32", 4)
    _check(cfg, 0.95, SWEEP, 10, 20, method=method, amplify=amplify)

CASES = [
    # m, n, r, c, k, dtype, S, steps, tolerance
    (10, 10, 5, 5, 2, "f32", 0.6, 6, 1),
    (192, 192, 32, 48, 5, "f32", 0.9, 8, 8),
    (200, 300, 100, 100, 4, "f16", 0.95, 10, 20),       # the LeNet-5 tile shape and rank
    (256, 512, 128, 256, 16, "bf16", 0.91, 9, 64),      # 4096-entry factors, several 64-column groups
    (64, 384, 32, 128, 40, "f16", 0.8, 7, 0),           # rank above 32, tolerance 0: mostly ineligible candidates
    (30, 77, 3, 7, 70, "bf16", 0.5, 5, 2),              # rank far above the tile size
]


@pytest.mark.parametrize("idx", range(len(CASES)))
def test_search_matches_the_oracle(idx):
    m, n, r, c, k, dtype, S, steps, tol = CASES[idx]
    _check(_cfg(m, n, r, c, k, dtype, 40 + idx), S, SWEEP, steps, tol)


def test_factors_beyond_on_chip_sort():
    """r k = 18000 entries: the sort runs in the workspace instead of on-chip memory."""
    _check(_cfg(600, 64, 600, 16, 30, "f16", 7), 0.9, [0.4, 0.8], 5, 100)


def test_paper_tile_shape():
    """576 x 512 tile at rank 145 (the ResNet-32 setting of Sec. 3): 83520 and 74240 factor entries."""
    _check(_cfg(576, 1024, 576, 512, 145, "bf16", 8, p=0.02), 0.7, [0.9, 0.97], 4, 3000)


def test_single_sp_and_single_step_degenerate_sweeps():
    cfg = _cfg(128, 128, 64, 64, 8, "f32", 9)
    _check(cfg, 0.9, [0.5], 1, 10)      # one candidate per tile: it wins whatever it is
    _check(cfg, 0.9, [1.0], 4, 10)      # I_p all zero: every probe keeps nothing
    _check(cfg, 0.9, [0.0, 1.0], 6, 10)


def test_repeated_calls_give_identical_bits_and_workspace_can_be_reused():
    cfg = _cfg(256, 512, 128, 256, 16, "f16", 10)
    d = desc_of(cfg)
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W = to_device(data["W"], cfg.dtype)
    t = lambda a: torch.from_numpy(a).to(dev())
    Mp, Mz = t(f["Mp"]), t(f["Mz"])
    ws = torch.empty(lrbi.search_workspace_bytes(d), dtype=torch.uint8, device=dev())
    ws.fill_(0xAB)
    a = lrbi.search_thresholds(d, W, f["w_threshold"], Mp, Mz, 0.9, SWEEP, 8, 50, workspace=ws)
    b = lrbi.search_thresholds(d, W, f["w_threshold"], Mp, Mz, 0.9, SWEEP, 8, 50, workspace=ws)
    c = lrbi.search_thresholds(d, W, f["w_threshold"], Mp, Mz, 0.9, SWEEP, 8, 50)
    torch.cuda.synchronize()
    for x, y, z in zip(a, b, c):
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int64),
                           y.view(torch.int32) if y.dtype == torch.float32 else y.view(torch.int64))
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int64),
                           z.view(torch.int32) if z.dtype == torch.float32 else z.view(torch.int64))


def test_full_size_layer_on_sampled_tiles():
    """C2 at full size, in the configuration the benchmark times: the oracle re-does the search on a few tiles."""
    cfg = workloads.CONFIGS["C2"]
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    W = to_device(data["W"], cfg.dtype)
    t = lambda a: torch.from_numpy(a).to(dev())
    S, sweep, steps, tol = 0.91, [0.88, 0.92, 0.95], 8, 64
    Tp, Tz, kept, cost = lrbi.search_thresholds(desc_of(cfg), W, f["w_threshold"], t(f["Mp"]), t(f["Mz"]), S, sweep,
                                                steps, tol)
    torch.cuda.synchronize()
    tile_cols = cfg.n // cfg.c
    rng = np.random.default_rng(5)
    for tile in sorted(rng.choice(cfg.tiles, size=6, replace=False).tolist()) + [0, cfg.tiles - 1]:
        ti, tj = divmod(tile, tile_cols)
        Wt = W64[ti * cfg.r:(ti + 1) * cfg.r, tj * cfg.c:(tj + 1) * cfg.c]
        rtp, rtz, rk, rc = alg1.search_thresholds(Wt, f["w_threshold"], f["Mp"][tile:tile + 1], f["Mz"][tile:tile + 1],
                                                  cfg.r, cfg.c, S, sweep, steps, tol)
        assert abs(float(cost[tile]) - rc[0]) <= 1e-12 * max(rc[0], 1.0)
        if float(Tp[tile]) == rtp[0] and float(Tz[tile]) == rtz[0]:
            assert int(kept[tile]) == int(rk[0])
        else:  # only a tie in cost may choose differently
            assert abs(int(kept[tile]) - round((1 - S) * cfg.r * cfg.c)) <= tol
