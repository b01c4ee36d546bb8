"""GPU parity of lrbi_nmf (Algorithm 1's first step, Sec. 2.1: non-negative factorisation of the magnitude matrix, tile
by tile; Sec. 3.2: weight-magnitude manipulation) against the oracle's float64 multiplicative updates."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import alg1
from oracle import nmf as nmf_oracle
from gpu_util import desc_of, dev, to_device

pytestmark = pytest.mark.gpu


def _cfg(m, n, r, c, k, dtype, seed):
    return workloads.Config("t", m, n, r, c, k, 0.1, 1, dtype, 0.05, seed)


def _start(cfg):
    rng = np.random.default_rng(cfg.seed + 500)
    T = cfg.tiles
    return (rng.uniform(0.1, 1.0, (T, cfg.r, cfg.k)).astype(np.float32),
            rng.uniform(0.1, 1.0, (T, cfg.k, cfg.c)).astype(np.float32))


def _check(cfg, iters, method=1, tol=2e-5):
    print("nmf", cfg, "iters", iters, "method", method, flush=True)
    data = workloads.make(cfg, want_x=False)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    Mp0, Mz0 = _start(cfg)
    thr = float(np.float32(1.6449 * cfg.sigma_w))
    S = 0.9
    amp = float(np.float32(1.0 / (1.0 - S)))
    Mp = torch.from_numpy(Mp0.copy()).to(dev())
    Mz = torch.from_numpy(Mz0.copy()).to(dev())
    lrbi.nmf(desc_of(cfg), to_device(data["W"], cfg.dtype), Mp, Mz, iters, eps=1e-9, method=method, w_threshold=thr,
             amplify=amp)
    torch.cuda.synchronize()
    # the oracle gets the amplification factor the library got (a float32), as 1 / (1 - S)
    S_eff = 1.0 - 1.0 / amp
    rp, rz = nmf_oracle.nmf(W64, Mp0, Mz0, cfg.r, cfg.c, iters, eps=1e-9, method=method, w_threshold=thr, S=S_eff)
    for got, ref, name in ((Mp.cpu().numpy(), rp, "Mp"), (Mz.cpu().numpy(), rz, "Mz")):
        scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))
        err = float(np.max(np.abs(got - ref) / scale))
        print("  %s max rel err %.3e" % (name, err), flush=True)
        assert err <= tol, (name, err)
        assert (got >= 0).all()
    return Mp, Mz


CASES = [
    # cfg, iterations, method
    (_cfg(10, 10, 5, 5, 2, "f32", 0), 5, 1),
    (_cfg(70, 90, 32, 40, 5, "f16", 1), 7, 2),            # cut-off tiles, odd number of iterations, squared magnitudes
    (_cfg(300, 520, 300, 260, 16, "bf16", 2), 6, 3),      # more rows / columns than one block of lanes; amplified
    (_cfg(128, 192, 64, 96, 40, "f32", 3), 4, 1),         # two register passes over the ranks
    (_cfg(1200, 64, 600, 64, 24, "f16", 4), 3, 1),        # several staged chunks of rows
    (_cfg(500, 800, 100, 100, 4, "f32", 5), 20, 1),       # the LeNet-5 layer shape, tile and rank
    (_cfg(512, 1024, 256, 256, 16, "f16", 6), 10, 1),     # the C2 tile shape and rank
    (_cfg(1024, 512, 512, 512, 32, "bf16", 7), 5, 1),     # the C3 tile shape and rank
    (_cfg(128, 128, 64, 64, 64, "f16", 8), 3, 1),
    (_cfg(576, 1024, 576, 512, 145, "bf16", 9), 3, 1),    # the paper's ResNet tile shape and rank (Sec. 4)
    (_cfg(576, 512, 576, 512, 256, "f16", 10), 2, 1),     # the largest rank of Table 1
    (_cfg(200, 136, 100, 68, 70, "f32", 11), 3, 2),       # rank above 64 with cut-off tiles and a ragged last pass
    (_cfg(640, 1300, 20, 40, 4, "f16", 12), 4, 1),        # 1056 tiles: more tiles than the chip needs, unsplit tiles
    (_cfg(2560, 5120, 256, 256, 16, "bf16", 13), 2, 3),   # 200 C2-shaped tiles... split; and
    (_cfg(5120, 6656, 256, 256, 12, "f16", 14), 2, 1),    # 520 of them: unsplit
]


@pytest.mark.parametrize("idx", range(len(CASES)))
def test_nmf_matches_the_oracle(idx):
    cfg, iters, method = CASES[idx]
    _check(cfg, iters, method)


def test_factorisation_then_search_end_to_end():
    """Algorithm 1 on the device, start to end: factorise |W|, search the thresholds, decode.  The factors come out
    of the library, the search result is checked against the oracle's search ON THOSE factors, and the objective has
    gone down."""
    cfg = _cfg(256, 512, 128, 128, 8, "f16", 11)
    data = workloads.make(cfg, want_x=False)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    W = to_device(data["W"], cfg.dtype)
    Mp0, Mz0 = _start(cfg)
    Mp = torch.from_numpy(Mp0.copy()).to(dev())
    Mz = torch.from_numpy(Mz0.copy()).to(dev())
    d = desc_of(cfg)
    lrbi.nmf(d, W, Mp, Mz, 30)
    torch.cuda.synchronize()
    mp, mz = Mp.cpu().numpy(), Mz.cpu().numpy()
    A = np.abs(W64)
    tile_cols = cfg.n // cfg.c
    for t in range(cfg.tiles):
        ti, tj = divmod(t, tile_cols)
        At = A[ti * cfg.r:(ti + 1) * cfg.r, tj * cfg.c:(tj + 1) * cfg.c]
        assert nmf_oracle.objective(At, mp[t], mz[t]) < 0.8 * nmf_oracle.objective(At, Mp0[t], Mz0[t])
    thr = float(np.float32(1.6449 * cfg.sigma_w))
    S, sweep, steps, tol = 0.9, [0.5, 0.7, 0.85], 8, 80
    Tp, Tz, kept, cost, ip, iz = lrbi.search_thresholds(d, W, thr, Mp, Mz, S, sweep, steps, tol, want_factors=True)
    mask = lrbi.decode_mask(d, ip.view(torch.int32), iz.view(torch.int32))
    torch.cuda.synchronize()
    rtp, rtz, rk, rc = alg1.search_thresholds(W64, thr, mp, mz, cfg.r, cfg.c, S, sweep, steps, tol)
    assert np.all(np.abs(cost.cpu().numpy() - rc) <= 1e-12 * np.maximum(rc, 1.0))
    same = (Tp.cpu().numpy() == rtp) & (Tz.cpu().numpy() == rtz)
    assert same.all() and np.array_equal(kept.cpu().numpy().astype(np.uint64), rk)
    # the decoded mask keeps exactly `kept` weights per tile
    from gpu_util import unpack_device_mask
    bits = unpack_device_mask(mask, cfg.n)[:, :cfg.n]
    for t in range(cfg.tiles):
        ti, tj = divmod(t, tile_cols)
        assert bits[ti * cfg.r:(ti + 1) * cfg.r, tj * cfg.c:(tj + 1) * cfg.c].sum() == int(kept[t])
